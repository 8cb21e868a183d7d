// Host-side launchers of the HIP kernels (internal to the library).
#pragma once
#include "common.hpp"

namespace aq {

// ---- quantizer block (quantize.hip)
aq_status launch_fill_u32(uint32_t* p, int n, uint32_t v, hipStream_t st);
// qdenom, qmax (largest unsigned code) and qw (largest symmetric code) describe the n-bit code range
aq_status launch_quantize_tensor(const float* d_w, int64_t rows, int64_t cols, int wscheme, float qdenom,
                                 int qmax, int qw, void* d_codes, float* d_scale, int32_t* d_zp, uint32_t* d_ws, hipStream_t st);
// The whole policy: activation parameters, weight ranges (per-tensor scheme), packed 8-bit weights and
// per-channel constants of every layer, in three or four launches.
aq_status launch_quantize_policy(const QTab* d_tab, const QTab& h_tab, const QPtrs& ptrs, const RangesArg& r,
                                 ActQ* actq, int* fast, int* status, uint32_t* mm, hipStream_t st);
// the quantize pass's traffic without its arithmetic (n a multiple of 4)
aq_status launch_stream_reference(const float* d_in, int64_t n, void* d_out, hipStream_t st);
// the pipelined wide kernel's k-step loop alone (mfma_reference.hip); sizes as in aq_mfma_loop_reference
aq_status launch_mfma_reference(const void* d_weights, const void* d_acts, int ksteps, bool stream_weights, int workgroups,
                                int32_t* d_acc, hipStream_t st);
aq_status launch_unpack_weights(const int8_t* wp, int N, int K, int KS, int asym, uint8_t* codes, hipStream_t st);

// ---- policy blob (quantize.hip): header words [0..15] = magic, version, hash lo/hi, payload bytes lo/hi, 0...
aq_status launch_blob_header_write(uint32_t* d_hdr, const uint32_t* h_words, hipStream_t st);
aq_status launch_blob_header_check(const uint32_t* d_hdr, const uint32_t* h_words, int* status, hipStream_t st);

// n-bit weight codes of one layer (operand order, signed domain) <-> sub-byte fields, 8 codes per n bytes
aq_status launch_pack_bits(const int8_t* wp, uint8_t* out, int64_t n_codes, int bits, int off, hipStream_t st);
aq_status launch_unpack_bits(const uint8_t* in, int8_t* wp, int64_t n_codes, int bits, int off, int N, int K, int KS,
                             hipStream_t st);

// ---- exploration on the produced actions (explore.hip)
aq_status launch_explore(void* d_actions, int64_t rows, int A, int head, const float* d_sigma, float epsilon,
                         uint64_t seed, uint64_t step, hipStream_t st);

// ---- 8-bit forward (forward_int8.hip)
struct FwdArgs {
    NetDev net;           // host copy, for planning
    const NetDev* d_net;  // the same, in device memory
    CallArgs c;
    TapArgs t;
    // host side only: per layer, the weights as nibbles for the few-row kernel (policies of at most 4 bits), or NULL
    const uint8_t* w4[AQ_MAX_LAYERS];
};

// whole-network fused MLP kernel; returns AQ_ESHAPE when the network does not fit it
bool any_taps(const FwdArgs& a);
bool fused_mlp_supported(const FwdArgs& a, int* rows_per_wg_out, size_t* lds_bytes_out, int* tiles_per_wave_out = nullptr);
aq_status launch_fused_mlp(const FwdArgs& a, hipStream_t st);
// software-pipelined whole-network kernel for wide layers (wide_mlp.hip); launch_fused_mlp hands it the shapes it takes
bool wide_mlp_supported(const FwdArgs& a, int* ld_out);
aq_status launch_wide_mlp(const FwdArgs& a, hipStream_t st);
// whole-network kernel for small networks, 16, 32 or 64 rows per workgroup (rows16_mlp.hpp / .hip);
// launch_fused_mlp hands it the shapes it takes
bool rows16_mlp_supported(const FwdArgs& a);
int rows16_mlp_row_tiles(int64_t batch);  // 16-row tiles per workgroup at this batch: 1, 2 or 4
bool rows16_mlp_alone_on_cu(int64_t batch);  // at most one 16-row workgroup per CU at this batch
aq_status launch_rows16_mlp(const FwdArgs& a, hipStream_t st);
// which kernel launch_fused_mlp runs for this network and batch (observations 16-byte aligned): 0 = the general
// fused kernel, 1 = the pipelined kernel for wide layers, 2 = the 16-row kernel for small networks
int fused_mlp_kernel_kind(const FwdArgs& a);

// one launch per layer (FC and implicit-GEMM convolution), activations in global memory
struct LayerIO {
    const void* in;   // layer 0: observations (fp32 or uint8); else int8 signed-domain [rows][K]
    int8_t* out;      // hidden layers: int8 signed-domain [rows][N] (row stride N)
    float* ln_x;      // LN layers: fp32 scratch [rows][N]
    float* y;         // last layer: dequantized outputs [rows][N]
};
aq_status launch_layer_int8(const FwdArgs& a, int layer, const LayerIO& io, hipStream_t st);
// FC layers at few rows: one workgroup per 32 x 32 output tile, K split over its waves (skinny_layer.hip)
bool skinny_layer_supported(const LayerDev& L, int64_t rows);
bool skinny_layer_does_argmax(const FwdArgs& a, int l);
// whether launch_layer_int8 hands layer l at this batch to the K-split kernel
// the leading convolution layers in one launch (0 layers = shapes it does not take); writes the last
// convolution's signed codes to `out` ([batch * oh * ow][N])
int conv_stack_layers(const FwdArgs& a);
aq_status launch_conv_stack(const FwdArgs& a, int8_t* out, hipStream_t st);
bool layer_uses_skinny(const FwdArgs& a, int l);
aq_status launch_layer_skinny(const FwdArgs& a, int l, const LayerIO& io, hipStream_t st);
// the few-row kernel's nibble weights from a layer's packed 8-bit operands: `pieces` = NT * KS * 64 (16 bytes -> 8)
aq_status launch_pack_nibbles(const int8_t* wp, uint8_t* w4, int64_t pieces, hipStream_t st);
aq_status launch_ln_tanh_rows(const FwdArgs& a, int layer, const float* x, int8_t* out, int64_t rows, hipStream_t st);
aq_status launch_head_rows(const float* y, int64_t rows, int N, int head, void* actions, hipStream_t st);

// ---- fp32 actor (forward_fp32.hip)
struct Fp32Layer {
    const float* w;
    const float* b;
    const float* gamma;
    const float* beta;
    int K, N, act;
    int in_h, in_w, in_c, kh, kw, stride, oh, ow;
};
aq_status launch_fp32_layer(const Fp32Layer& L, const void* in, int in_u8, float* out, int64_t rows, int relu,
                            hipStream_t st);
aq_status launch_fp32_ln_tanh(float* x, int64_t rows, int N, const float* gamma, const float* beta, float eps,
                              hipStream_t st);
aq_status launch_fp32_head(const float* y, int64_t rows, int N, int head, void* actions, hipStream_t st);
aq_status launch_init_keys(uint32_t* keys, int n_pairs, hipStream_t st);
aq_status launch_minmax_keys(const void* x, int is_u8, int64_t n, uint32_t* keys, hipStream_t st);
aq_status launch_keys_to_ranges(const uint32_t* keys, int n, float* out, hipStream_t st);


// ---- half-precision actor (fp16_actor.hip)
struct Fp16Layer {
    const void* wp;     // binary16 weights in MFMA operand order, [NT][KS16] tiles of 1 KiB
    const float* bias;  // binary16 values widened to fp32, padded to NT * 32
    int K, N, KS16, NT, fc, relu;
    int in_h, in_w, in_c, kh, kw, stride, oh, ow;
    float* head_actions;  // last layer with an elementwise head: fp32 actions [rows][N], else NULL
    int head_tanh;
    int32_t* head_argmax;  // last layer of an argmax policy run by the few-row kernel with one feature tile:
                           // action indices [rows], else NULL
};
aq_status launch_fp16_pack_weights(const float* w, int N, int K, int KS16, int NT, void* wp, int* status,
                                   hipStream_t st);
aq_status launch_fp16_round_vec(const float* src, int n, int n_pad, float fill, float* dst, int* status,
                                hipStream_t st);
// in_mode: 0 = binary16 activations, 1 = fp32 observations, 2 = uint8 observations
aq_status launch_layer_fp16(const Fp16Layer& L, const void* in, int in_mode, void* out, int64_t rows,
                            hipStream_t st);
// whether launch_layer_fp16 takes the few-row (K-split) kernel for this layer
bool fp16_layer_is_skinny(const Fp16Layer& L, const void* in, int in_mode, int64_t rows);
aq_status launch_fp16_ln_tanh(void* x, int64_t rows, int N, const float* gamma, const float* beta, float eps,
                              hipStream_t st);
aq_status launch_fp16_head(const void* y, int64_t rows, int N, int head, void* actions, hipStream_t st);
// the leading convolutions of a frame policy in one launch (fp16_conv_stack.hip): how many layers it takes
// (0 = none of these shapes), and the launch, which writes the last convolution's map to `out`
int fp16_conv_stack_layers(const Fp16Layer* L, int n_layers, const void* obs, int in_mode0, int64_t batch);
aq_status launch_fp16_conv_stack(const Fp16Layer* L, int n_layers, const void* obs, int in_mode0, int64_t batch,
                                 void* out, hipStream_t st);

}  // namespace aq
