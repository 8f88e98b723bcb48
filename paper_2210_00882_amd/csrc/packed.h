// Layout of network parameters re-ordered for the MFMA kernels ("packed"
// parameters), shared by the packing kernel and the rollout kernels.
//
// The rollout kernels compute every layer transposed: out^T = W^T * in^T, so the
// weights are the MFMA "A" operand (32 output units x k input units per
// instruction), the batch rows are the 32 columns of the "B" operand, and a
// layer's result lands in the accumulator layout
//     lane (n = lane % 32, h = lane / 32), register r  <->  row n, unit 8*(r/4) + 4*h + r%4.
// Because the order of the k index inside a contraction is free, the weights of
// the next layer are stored so that this accumulator layout can be fed straight
// back in as the next B operand, with no transpose through LDS ("chained" map).
//
// A tile is 1 KiB: 64 lanes x 16 bytes; lane (m = lane % 32, h) holds, for output
// unit 32*uc + m, the inputs
//   bf16 : 8 values s = 0..7  = the k slots 8*h + s of one 32x32x16 MFMA
//   f32  : 4 values j = 0..3  = the k slot h of four consecutive 32x32x2 MFMAs.
// Input index of (tile kt, h, s or j):
//   chained bf16 : 32*(kt/2) + 16*(kt%2) + 8*(s/4) + 4*h + s%4
//   chained f32  : 32*(kt/4) + 8*(kt%4) + 4*h + j
//   linear  bf16 : 16*kt + 8*h + s                  (particle observation, layer 1)
//   pairs   f32  : 8*kt + 2*j + h                   (particle observation, layer 1)
// Inputs or outputs beyond the real sizes hold zeros.
//
// Biases of layers 1 and 2 ride along as one more input: input index n_in holds
// the bias, and the kernels feed the constant 1 at that index.  (A bias read
// from LDS costs as much LDS bandwidth per chunk as four weight tiles; one more
// MFMA is cheaper.)  For layer 1 the index falls into the padding of the last
// tile when there is room, for layer 2 it opens one extra tile.
//
// One network (two hidden layers) =
//   [layer-1 tiles (uc major, kt minor), nuc * kt1 tiles, kt1 = tiles(in_used + 1)]
//   [chunk block uc = 0 .. nuc-1], each kt2 + 1 + 2 tpc tiles:
//       kt2 layer-2 tiles of the 32-unit chunk uc, 1 bias tile of chunk uc,
//       tpc = kt2/nuc layer-3 tiles that consume the outputs of chunk uc-1
//       (zeros for uc = 0), tpc layer-3 tiles that consume the outputs of chunk uc
//   [b3: 32 floats in physical output order]
// With more than two hidden layers, every further hidden layer contributes nuc chunk blocks of the
// same size in front of those of the last hidden layer (layer order), with the layer-3 slots unused.
// The kernels keep the layer-1 tiles resident in LDS and stream the chunk blocks
// through an LDS window, one block per stage; they activate chunk uc-1 while the
// MFMAs of chunk uc run, which is why a block carries the layer-3 tiles of the
// chunk before it (the copy for chunk uc itself is used after the last block).
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace msrl {

enum InMap : int { IN_CHAIN = 0, IN_LINEAR16 = 1, IN_PAIRS = 2 };
// physical output row m of a layer-3 tile -> logical output
//   OUT_NATURAL : m
//   OUT_GAUSS   : m < 8 -> mean m;  8 <= m < 16 -> log-std (m - 8)   (act_dim <= 8)
enum OutMap : int { OUT_NATURAL = 0, OUT_GAUSS = 1 };

struct NetLayout {
  int kt1, kt2, nuc, tpc;  // tiles per chunk in layer 1 / layer 2; chunks of 32 units; layer-3 tiles per chunk
  int chunk_tiles;         // tiles of one chunk block
  int layers;              // hidden layers (>= 2); chunk blocks: (layers - 1) * nuc
  size_t w1;               // byte offset of the layer-1 tiles
  size_t chunks;           // byte offset of chunk block 0
  size_t chunk_bytes;      // size of one chunk block
  size_t b3;               // byte offset of the output bias
  size_t bytes;            // size of one packed network, a multiple of 1 KiB
};

__host__ __device__ inline int tiles_for_inputs(int n_in, bool bf16) {
  return bf16 ? (n_in + 15) / 16 : (n_in + 7) / 8;
}

// in_used: number of leading inputs of layer 1 that are packed (the rest are known to be zero)
__host__ __device__ inline NetLayout net_layout(int in_used, int hidden, bool bf16, int layers = 2) {
  NetLayout L;
  L.kt1 = tiles_for_inputs(in_used + 1, bf16);
  L.kt2 = tiles_for_inputs(hidden, bf16);
  L.nuc = hidden / 32;
  L.tpc = L.kt2 / L.nuc;
  L.chunk_tiles = L.kt2 + 1 + 2 * L.tpc;
  L.layers = layers;
  L.w1 = 0;
  L.chunks = L.w1 + (size_t)L.nuc * L.kt1 * 1024;
  L.chunk_bytes = (size_t)L.chunk_tiles * 1024;
  L.b3 = L.chunks + (size_t)(layers - 1) * L.nuc * L.chunk_bytes;
  L.bytes = (L.b3 + 32 * 4 + 1023) / 1024 * 1024;
  return L;
}

// One matrix (or bias vector) to re-order.
struct PackJob {
  const void* src;    // device
  const void* bias;   // device, or null: values served at input index bias_index
  void* dst;          // device
  int src_bf16;       // source element type (dst tiles have the same type; bias vectors become f32)
  int is_bias;        // 1: copy n_out values through the output map into 32*nuc floats
  int n_in, n_out;    // logical sizes
  int bias_index;     // input index that reads bias[out] (only if bias != null)
  int src_out_major;  // 0: src[in * n_out + out] (network weights); 1: src[out * n_in + in]
  int nuc, kt;        // output chunks, tiles per chunk
  // destination tile of (output chunk uc, input tile kt):
  //   (uc + kt / group) * chunk_stride + slot_base + kt % group
  // layers 1, 2: group = kt (tiles of a chunk are consecutive); layer 3: group = tiles
  // per chunk block, so its tiles follow the layer-2 tiles of the chunk they consume.
  int group, chunk_stride, slot_base;
  int in_map, out_map, gauss_k;
  // in_block > 0: the packed inputs come in blocks of in_block; input i reads source input
  // (i / in_block) * in_block_stride + i % in_block if i % in_block < in_block_used and is zero otherwise
  // (the joint observation of a centralised critic: per agent, the non-zero prefix of its row padded to
  // whole tiles; the bias sits in the padding of the first block, at bias_index)
  int in_block, in_block_used, in_block_stride;
  // fp32 images: factor on the weights and on the bias riding with them (1, or TANH_PRESCALE for the layers
  // that end in tanh); bf16 images are not scaled (the product would not be a bfloat16 value)
  float scale;
};

struct PackJobs {
  int n;
  PackJob job[24];
};

}  // namespace msrl
