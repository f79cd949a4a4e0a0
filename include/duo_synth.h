/*
 * duo_synth.h - device twin of the seeded, position-addressable input generator
 * (libduosynth.so).  Test and benchmark infrastructure only: it produces the
 * synthetic bf16 N(0,1) Q/K/V tensors that stand in for real activations, with
 * exactly the bits of the CPU generator, so multi-gigabyte caches can be filled
 * on the device while the CPU regenerates any slice it wants to check.
 * Holds none of the attention method's arithmetic.
 */
#ifndef DUO_SYNTH_H
#define DUO_SYNTH_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* dst: DEVICE bf16 [n_pos][n_heads][head_dim] for positions pos_start .. pos_start+n_pos-1.
 * table: DEVICE uint16[65536], bf16 bits of the standard-normal quantiles.
 * key: the 64-bit stream key of (seed, layer, tensor, sequence).
 * Element (pos, head, d) with counter c = (pos*n_heads + head)*head_dim + d gets
 * table[mix64(key ^ (c * 0x9E3779B97F4A7C15)) >> 48], mix64 being two
 * xor-shift/multiply rounds and a final xor-shift.
 * Returns 0, or -1 for bad arguments, -5 if the launch failed. */
int duo_synth_fill_bf16(void* dst, const uint16_t* table, uint64_t key, int64_t pos_start,
                        int64_t n_pos, int32_t n_heads, int32_t head_dim, void* stream);

#ifdef __cplusplus
}
#endif
#endif
