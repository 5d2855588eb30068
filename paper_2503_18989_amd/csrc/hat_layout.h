// Memory layouts shared by all kernels of the middle-submodel forward.
//
// (1) "P32" operand layout.  Every GEMM operand -- re-tiled weights and all
//     activations, both fp16 (act_t) -- is stored as panels of 32 rows; inside a panel the unit is
//     an "octet" (8 consecutive k elements of one row, 16 bytes) and octets are
//     ordered [k/8][row%32].  A lane of a 64-wide wavefront that needs MFMA
//     32x32x16 operand rows (lane%32) and k-octet (lane/32) therefore reads
//     16 bytes at lane*16 from a 1 KB block: global loads are fully coalesced and
//     LDS reads are conflict-free, with no swizzle.
//       element (r, k) of an [R, K] matrix, K % 8 == 0:
//         ((r/32) * (K/8) + k/8) * 256 + (r%32) * 8 + k%8
//
// (2) KV pool.  pool[layer][head][page] = one K tile followed by one V tile, each
//     16 tokens x head_dim bf16 (a device's consecutively allocated pages are one
//     contiguous run per head).
//       K tile: [hd/8][slot][8]                   (an octet-major 16-row panel)
//       V tile: [hd/32][h][hd%32][j], where slot = 8*(j/4) + 4*h + j%4
//     The V order is the order in which a lane of the S^T = K Q^T accumulator
//     holds its keys, so softmax probabilities feed the P*V MFMA from registers.
#pragma once
#include <stdint.h>

#define HAT_HOSTDEV __host__ __device__ __forceinline__

HAT_HOSTDEV size_t p32_index(int r, int k, int K) {
  return ((size_t)(r >> 5) * (size_t)(K >> 3) + (size_t)(k >> 3)) * 256 + (size_t)((r & 31) * 8 + (k & 7));
}

// element offsets inside one K / V tile
HAT_HOSTDEV int ktile_index(int slot, int hd_i) { return (hd_i >> 3) * 128 + slot * 8 + (hd_i & 7); }
HAT_HOSTDEV int vtile_index(int slot, int hd_i) {
  int h = (slot >> 2) & 1;
  int j = ((slot >> 3) << 2) | (slot & 3);
  return (hd_i >> 5) * 512 + h * 256 + (hd_i & 31) * 8 + j;
}

// elements of one (page, head) record: K tile + V tile
HAT_HOSTDEV size_t kv_head_elems(int head_dim) { return (size_t)2 * 16 * head_dim; }
HAT_HOSTDEV size_t kv_page_elems(int n_heads, int head_dim) { return (size_t)n_heads * kv_head_elems(head_dim); }
