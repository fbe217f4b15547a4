/*
 * CPU oracle for the KV-migration hot path: TEST INFRASTRUCTURE ONLY.
 *
 * Plain nested loops that write out, one byte at a time, which byte of a
 * source paged-KV pool ends up where after a tensor-parallel switch
 * (paper Sec. 3.2.2, "Aggregated and Pipelined KV Migration": KV is split
 * evenly over the GPUs of a TP group along the head dimension, and the
 * migration kernel first gathers the scattered per-page regions of the moved
 * head slice into one contiguous buffer).  Aggregation, double buffering and
 * pipelining only change the schedule, never the bytes, so the oracle is the
 * definition itself.  Nothing here is shared with, or derived from, the HIP
 * path; only tests, the smoke check and the bench's cpu_baseline leg use it.
 *
 * Pool layout (the paper does not fix one; this is the reading used by the
 * whole build): pool[l][c][slot][head][x], l < L layers, c = 0 for K and 1
 * for V, slot < S token slots, head < H_local heads held by this GPU,
 * x < D elements of `e` bytes.  Stream layout: stream[l][c][j][h][x] with
 * j < T the flattened token index and h < w the heads of the moved slice.
 *
 * Pins: tests/test_oracle_pins.py (library gather/scatter reduction,
 * dictionary brute force, identity and permutation special cases, sentinel
 * invariant, paper's size identity).
 */
#include <stddef.h>
#include <stdint.h>

/* gather: stream[l][c][j][h][x] = src[l][c][sslot[j]][src_head_off+h][x] */
void orc_pack(const uint8_t *src, int64_t L, int64_t S, int64_t Hs, int64_t D, int64_t e,
              const int32_t *sslot, int64_t T, int64_t src_head_off, int64_t w,
              uint8_t *stream)
{
    for (int64_t l = 0; l < L; ++l)
        for (int64_t c = 0; c < 2; ++c)
            for (int64_t j = 0; j < T; ++j)
                for (int64_t h = 0; h < w; ++h)
                    for (int64_t x = 0; x < D; ++x)
                        for (int64_t b = 0; b < e; ++b) {
                            int64_t si = ((((l * 2 + c) * S + sslot[j]) * Hs + (src_head_off + h)) * D + x) * e + b;
                            int64_t ti = ((((l * 2 + c) * T + j) * w + h) * D + x) * e + b;
                            stream[ti] = src[si];
                        }
}

/* scatter: dst[l][c][dslot[j]][dst_head_off+h][x] = stream[l][c][j][h][x]; other bytes untouched */
void orc_unpack(const uint8_t *stream, int64_t L, int64_t S, int64_t Hd, int64_t D, int64_t e,
                const int32_t *dslot, int64_t T, int64_t dst_head_off, int64_t w,
                uint8_t *dst)
{
    for (int64_t l = 0; l < L; ++l)
        for (int64_t c = 0; c < 2; ++c)
            for (int64_t j = 0; j < T; ++j)
                for (int64_t h = 0; h < w; ++h)
                    for (int64_t x = 0; x < D; ++x)
                        for (int64_t b = 0; b < e; ++b) {
                            int64_t ti = ((((l * 2 + c) * T + j) * w + h) * D + x) * e + b;
                            int64_t di = ((((l * 2 + c) * S + dslot[j]) * Hd + (dst_head_off + h)) * D + x) * e + b;
                            dst[di] = stream[ti];
                        }
}

/* the migration written directly, never forming the stream */
void orc_migrate_direct(const uint8_t *src, int64_t S_src, int64_t Hs, int64_t src_head_off,
                        uint8_t *dst, int64_t S_dst, int64_t Hd, int64_t dst_head_off,
                        int64_t L, int64_t D, int64_t e, int64_t w,
                        const int32_t *sslot, const int32_t *dslot, int64_t T)
{
    for (int64_t l = 0; l < L; ++l)
        for (int64_t c = 0; c < 2; ++c)
            for (int64_t j = 0; j < T; ++j)
                for (int64_t h = 0; h < w; ++h)
                    for (int64_t x = 0; x < D; ++x)
                        for (int64_t b = 0; b < e; ++b) {
                            int64_t si = ((((l * 2 + c) * S_src + sslot[j]) * Hs + (src_head_off + h)) * D + x) * e + b;
                            int64_t di = ((((l * 2 + c) * S_dst + dslot[j]) * Hd + (dst_head_off + h)) * D + x) * e + b;
                            dst[di] = src[si];
                        }
}
