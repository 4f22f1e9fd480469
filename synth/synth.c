/*
 * Seeded synthetic-input generator, host side (harness code).
 *
 * Holds none of the decode method's arithmetic: it only turns (seed, tensor id,
 * flat index) into a table slot through an integer hash. The table of bf16 bit
 * patterns (normal quantiles scaled to the requested mean / sigma) is built by
 * the Python side and passed in. The device-side generator (synth/gpu.py)
 * evaluates the same hash with torch integer ops; the two must agree bit for
 * bit, which tests/test_synth.py checks.
 *
 * Hash: two rounds of the murmur3 32-bit finaliser (a published mixing
 * function) keyed by two 32-bit keys derived from (seed, tensor id).
 */
#include <stdint.h>
#include <stddef.h>

static inline uint32_t fmix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85ebca6bu;
    h ^= h >> 13;
    h *= 0xc2b2ae35u;
    h ^= h >> 16;
    return h;
}

uint32_t synth_hash(uint32_t key1, uint32_t key2, uint32_t idx)
{
    return fmix32(fmix32(idx ^ key1) + key2);
}

/* out_bits[i] = table[hash(i0 + i) & 0xFFFF], bf16 bit patterns. */
void synth_fill_bf16(uint16_t *out_bits, int64_t n, int64_t i0, uint32_t key1, uint32_t key2,
                     const uint16_t *table)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out_bits[i] = table[synth_hash(key1, key2, (uint32_t)(i0 + i)) & 0xFFFFu];
}

/* Same values widened exactly to fp32 (bf16 bits << 16). */
void synth_fill_f32(float *out, int64_t n, int64_t i0, uint32_t key1, uint32_t key2,
                    const uint16_t *table)
{
    uint32_t *o = (uint32_t *)out;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        o[i] = (uint32_t)table[synth_hash(key1, key2, (uint32_t)(i0 + i)) & 0xFFFFu] << 16;
}

/* Fills selected blocks of a tensor that is laid out in full at `out`: block b covers the
 * elements [b * block_elems, (b + 1) * block_elems).  Other elements are left untouched. */
void synth_fill_f32_blocks(float *out, const int32_t *blocks, int64_t n_blocks, int64_t block_elems,
                           uint32_t key1, uint32_t key2, const uint16_t *table)
{
    uint32_t *o = (uint32_t *)out;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_blocks; ++j) {
        int64_t base = (int64_t)blocks[j] * block_elems;
        for (int64_t i = 0; i < block_elems; ++i)
            o[base + i] = (uint32_t)table[synth_hash(key1, key2, (uint32_t)(base + i)) & 0xFFFFu] << 16;
    }
}
