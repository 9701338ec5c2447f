// Measurement aids (include/zi_probe.h): HBM stream probe, host-link probe, storage probe.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstring>

#include "zi_engine_internal.h"
#include "zi_probe.h"

using namespace zi::host;

extern "C" zi_status zi_hbm_probe(void* d_a, void* d_b, size_t bytes, int32_t mode, void* hip_stream)
{
    if (mode < 0 || mode > 2) return fail(ZI_ERR_INVALID_ARG, "mode must be 0 (read), 1 (copy) or 2 (in-place update)");
    if (!d_a) return fail(ZI_ERR_INVALID_ARG, "d_a is NULL");
    if (mode == 1 && !d_b) return fail(ZI_ERR_INVALID_ARG, "d_b is NULL");
    if (bytes < 16 || bytes % 16) return fail(ZI_ERR_INVALID_ARG, "bytes must be a positive multiple of 16");
    if (bytes / 16 / 256 >= 0x7FFFFFFFull) return fail(ZI_ERR_INVALID_ARG, "bytes too large for one launch");
    if (!aligned(d_a, 16) || !aligned(d_b, 16)) return fail(ZI_ERR_ALIGNMENT, "buffers must be 16-byte aligned");
    if (zi_status st = check_kernel_visible(d_a, bytes, -1, "d_a")) return st;
    if (mode == 1)
        if (zi_status st = check_kernel_visible(d_b, bytes, -1, "d_b")) return st;
    // mode 0 needs a place for a store that never happens: the first float of d_a itself
    ZI_HIP(zi::launch_hbm_probe(d_a, d_b, (int64_t)(bytes / 16), mode, (float*)d_a, (hipStream_t)hip_stream));
    return ZI_OK;
}

extern "C" zi_status zi_engine_link_probe(zi_engine* e, const void* host_src, void* host_dst, size_t bytes,
                                          int32_t mode, size_t piece_bytes, int32_t depth, double* seconds_out)
{
    if (zi_status st = check_engine(e)) return st;
    if (mode < 0 || mode > 2) return fail(ZI_ERR_INVALID_ARG, "mode must be 0, 1 or 2");
    if (depth < 0 || depth > 8) return fail(ZI_ERR_INVALID_ARG, "depth must be in 0..8 (0 = no limit)");
    if (!seconds_out) return fail(ZI_ERR_INVALID_ARG, "seconds_out is NULL");
    if ((mode == 0 || mode == 2) && !host_src) return fail(ZI_ERR_INVALID_ARG, "host_src is NULL");
    if ((mode == 1 || mode == 2) && !host_dst) return fail(ZI_ERR_INVALID_ARG, "host_dst is NULL");
    if (bytes == 0) return fail(ZI_ERR_INVALID_ARG, "bytes is 0");
    const size_t half = (size_t)e->n_slots * kSlotArrays * e->array_bytes / 2 / 4096 * 4096;
    if (piece_bytes == 0) piece_bytes = e->chunk_bytes;
    if (piece_bytes > half) return fail(ZI_ERR_INVALID_ARG, "piece_bytes above half of the staging memory (%zu)", half);
    if (mode != 1 && memory_kind(host_src) != 1) return fail(ZI_ERR_INVALID_ARG, "host_src must be pinned host memory");
    if (mode != 0 && memory_kind(host_dst) != 1) return fail(ZI_ERR_INVALID_ARG, "host_dst must be pinned host memory");
    ZI_HIP(hipSetDevice(e->device));
    ZI_HIP(hipStreamSynchronize(e->s_h2d));
    ZI_HIP(hipStreamSynchronize(e->s_d2h));

    // Host-to-device pieces land in the first half of the staging memory, device-to-host pieces leave
    // from the second half, so the two directions never touch the same staging bytes.  Pieces in flight
    // in one direction use different parts of their half while there is room.
    const size_t rooms = half / piece_bytes;              // >= 1
    char* const in_base = e->staging;
    char* const out_base = e->staging + half;
    const auto t0 = std::chrono::steady_clock::now();
    int64_t piece = 0;
    for (size_t off = 0; off < bytes; off += piece_bytes, ++piece) {
        const size_t nb = bytes - off < piece_bytes ? bytes - off : piece_bytes;
        const int ev = (int)(piece % 8);
        if (depth > 0 && piece >= depth) {
            const int old = (int)((piece - depth) % 8);
            if (mode != 1) ZI_HIP(hipEventSynchronize(e->ev_h2d[old]));
            if (mode != 0) ZI_HIP(hipEventSynchronize(e->ev_d2h[old]));
        }
        const size_t room = (size_t)(piece % (int64_t)rooms) * piece_bytes;
        if (mode != 1) {
            ZI_HIP(hipMemcpyAsync(in_base + room, (const char*)host_src + off, nb, hipMemcpyHostToDevice, e->s_h2d));
            if (depth > 0) ZI_HIP(hipEventRecord(e->ev_h2d[ev], e->s_h2d));
        }
        if (mode != 0) {
            ZI_HIP(hipMemcpyAsync((char*)host_dst + off, out_base + room, nb, hipMemcpyDeviceToHost, e->s_d2h));
            if (depth > 0) ZI_HIP(hipEventRecord(e->ev_d2h[ev], e->s_d2h));
        }
    }
    ZI_HIP(hipStreamSynchronize(e->s_h2d));
    ZI_HIP(hipStreamSynchronize(e->s_d2h));
    *seconds_out = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return ZI_OK;
}

extern "C" zi_status zi_engine_file_probe(zi_engine* e, int32_t fd_read, int32_t fd_write, size_t bytes,
                                          double* seconds_out)
{
    ZI_GUARD_BEGIN
    if (zi_status st = check_engine(e)) return st;
    if (!seconds_out) return fail(ZI_ERR_INVALID_ARG, "seconds_out is NULL");
    if (e->n_hslots == 0) return fail(ZI_ERR_INVALID_ARG, "the probe needs a pinned ring (ZI_OPT_HOST_RING_SLOTS)");
    if (fd_read < 0 && fd_write < 0) return fail(ZI_ERR_INVALID_ARG, "no file descriptor given");
    if (bytes == 0 || bytes % 4096) return fail(ZI_ERR_INVALID_ARG, "bytes must be a positive multiple of 4096");
    if (e->n_hslots < 2) return fail(ZI_ERR_INVALID_ARG, "ring too small");
    // Reads land in the first half of the ring, writes leave from the second half.
    const size_t half = (size_t)(e->n_hslots / 2) * kSlotArrays * e->array_bytes / 4096 * 4096;
    auto pieces_for = [&](int fd, int op, char* base, std::vector<Piece>& out) {
        const int fl = fcntl(fd, F_GETFL);
        const bool direct = fl >= 0 && (fl & O_DIRECT);
        size_t ring_o = 0;
        out.clear();
        for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
            const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
            if (ring_o + nb > half) ring_o = 0;
            out.push_back({op, base + ring_o, nullptr, fd, (int64_t)o, nb, nb, direct});
            ring_o += nb;
        }
    };
    e->pieces_in.clear();
    e->pieces_out.clear();
    if (fd_read >= 0) pieces_for(fd_read, 1, e->hring, e->pieces_in);
    if (fd_write >= 0) pieces_for(fd_write, 2, e->hring + half, e->pieces_out);
    struct Writer {
        zi_engine* e;
        int err;
        static void main(void* ctx)
        {
            Writer& w = *static_cast<Writer*>(ctx);
            w.err = run_pieces(*w.e->pool_out, w.e->pieces_out);
        }
    } writer{e, 0};
    int err_r = 0;
    const auto t0 = std::chrono::steady_clock::now();
    if (!e->pieces_out.empty()) e->stage_out->start(&Writer::main, &writer);
    if (!e->pieces_in.empty()) err_r = run_pieces(*e->pool_in, e->pieces_in);
    if (!e->pieces_out.empty()) e->stage_out->wait();
    *seconds_out = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    if (err_r) return fail(ZI_ERR_IO, "reading: %s", strerror(err_r));
    if (writer.err) return fail(ZI_ERR_IO, "writing: %s", strerror(writer.err));
    return ZI_OK;
    ZI_GUARD_END
}
