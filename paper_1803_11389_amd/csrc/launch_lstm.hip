// Host side of the LSTM comparator (kernel_lstm.hip.h): argument checks, workspace layout and the
// launch sequence of Section 3.1 of arXiv 1803.11389 -- per block and layer one pass over W for the
// input products of the block's steps, then one pass over U per time step.
#include "host.hip.h"
#include "kernel_lstm.hip.h"

namespace ssrnn {

namespace {

constexpr size_t LSTM_ALIGN = 256;
size_t lstm_align_up(size_t v) { return (v + LSTM_ALIGN - 1) / LSTM_ALIGN * LSTM_ALIGN; }

struct LstmLayout {
  size_t hstate_offset, hstate_stride;   // two copies of the layers' h_{t-1} ([n_layers x d]), read and written in turn
  size_t g_offset;                       // input products of one block: [block x 4d]
  size_t act_offset, act_stride;         // two hand-off buffers [block x d] between layers
  size_t total;
};

LstmLayout lstm_layout(int n_layers, int d, int block) {
  LstmLayout l{};
  size_t off = 0;
  l.hstate_offset = off;
  l.hstate_stride = lstm_align_up(static_cast<size_t>(n_layers) * d * sizeof(float));
  off += 2 * l.hstate_stride;
  l.g_offset = off;
  off += lstm_align_up(static_cast<size_t>(block) * 4 * d * sizeof(float));
  l.act_offset = off;
  l.act_stride = lstm_align_up(static_cast<size_t>(block) * d * sizeof(float));
  off += 2 * l.act_stride;
  l.total = off;
  return l;
}

bool lstm_shape_ok(int n_layers, int d, int T) {
  return n_layers >= 1 && n_layers <= 4096 && d >= 1 && d <= (1 << 16) && T >= 1;
}

int lstm_block(int T) { return T < LSTM_MAX_TT ? T : LSTM_MAX_TT; }

bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

__global__ void lstm_init_kernel(const float* src, float* dst, long n) {
  const long i = blockIdx.x * static_cast<long>(blockDim.x) + threadIdx.x;
  if (i < n) dst[i] = src ? src[i] : 0.0f;
}

template <bool VEC>
int launch_input(const float* W, const float* bias, const float* x, long ldx, float* G, int nt, int d, hipStream_t st) {
  const int groups = (d + LSTM_WAVES - 1) / LSTM_WAVES;
  const dim3 grid(groups < 8192 ? groups : 8192), block(LSTM_WAVES * 64);
#define SSRNN_LSTM_IN(TT_)                                                                          \
  if (nt <= TT_) {                                                                                  \
    hipLaunchKernelGGL((lstm_input_kernel<TT_, VEC>), grid, block, 0, st, W, bias, x, ldx, G, nt, d); \
    return SSRNN_OK;                                                                                \
  }
  SSRNN_LSTM_IN(1) SSRNN_LSTM_IN(2) SSRNN_LSTM_IN(4) SSRNN_LSTM_IN(8) SSRNN_LSTM_IN(16)
#undef SSRNN_LSTM_IN
  return fail(SSRNN_EUNSUPPORTED, "lstm_forward: %d steps in one pass over W", nt);
}

// Waves per workgroup of the step kernel.  A wave takes one feature at a time, so there are d / waves
// workgroups; the count (at least four) for which the busiest of the 256 compute units walks the fewest
// features: rounds of workgroups times features per workgroup.
int lstm_step_waves(int d) {
  int best = 4;
  long best_walks = -1;
  for (int nw = 4; nw <= LSTM_STEP_MAX_WAVES; ++nw) {
    const long groups = (d + nw - 1) / nw;
    const long walks = (groups + 255) / 256 * nw;
    if (best_walks < 0 || walks < best_walks) { best_walks = walks; best = nw; }
  }
  return best;
}

}  // namespace

size_t lstm_workspace_bytes_impl(int n_layers, int d, int T) {
  if (!lstm_shape_ok(n_layers, d, T)) return 0;
  return lstm_layout(n_layers, d, lstm_block(T)).total;
}

int lstm_forward_impl(const float* const* W, const float* const* U, const float* const* bias, const float* x,
                      const float* h_init, const float* c_init, float* h, float* h_final, float* c_final,
                      int n_layers, int d, long L, int T, int flags, void* workspace, size_t workspace_bytes,
                      void* stream) {
  if (!W || !U) return fail(SSRNN_EINVAL, "lstm_forward: W or U is NULL");
  if (!h_final || !c_final) return fail(SSRNN_EINVAL, "lstm_forward: h_final or c_final is NULL");
  if (n_layers < 1 || d < 1 || L < 0 || T < 1) return fail(SSRNN_EINVAL, "lstm_forward: n_layers %d, d %d, L %ld, T %d", n_layers, d, L, T);
  if (flags != 0) return fail(SSRNN_EINVAL, "lstm_forward: flags must be 0");
  if (!lstm_shape_ok(n_layers, d, T)) return fail(SSRNN_EUNSUPPORTED, "lstm_forward: shape out of range (n_layers %d, d %d)", n_layers, d);
  if (L > 0 && (!x || !h)) return fail(SSRNN_EINVAL, "lstm_forward: x or h is NULL");
  for (int l = 0; l < n_layers; ++l)
    if (!W[l] || !U[l]) return fail(SSRNN_EINVAL, "lstm_forward: W[%d] or U[%d] is NULL", l, l);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long nstate = static_cast<long>(n_layers) * d;
  const int block = lstm_block(L > 0 && L < T ? static_cast<int>(L) : T);
  const LstmLayout wl = lstm_layout(n_layers, d, block);
  if (L > 0) {
    if (!workspace) return fail(SSRNN_EINVAL, "lstm_forward: workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) % LSTM_ALIGN) return fail(SSRNN_EINVAL, "lstm_forward: workspace must be 256-byte aligned");
    if (workspace_bytes < wl.total) return fail(SSRNN_EWORKSPACE, "lstm_forward: workspace of %zu bytes, %zu needed", workspace_bytes, wl.total);
  }
  const dim3 sg(static_cast<unsigned>((nstate + 255) / 256)), sb(256);
  if (c_final != c_init) hipLaunchKernelGGL(lstm_init_kernel, sg, sb, 0, st, c_init, c_final, nstate);
  if (L == 0) {
    if (h_final != h_init) hipLaunchKernelGGL(lstm_init_kernel, sg, sb, 0, st, h_init, h_final, nstate);
    HIP_TRY(hipGetLastError());
    return SSRNN_OK;
  }
  char* ws = static_cast<char*>(workspace);
  float* hstate[2] = {reinterpret_cast<float*>(ws + wl.hstate_offset), reinterpret_cast<float*>(ws + wl.hstate_offset + wl.hstate_stride)};
  float* G = reinterpret_cast<float*>(ws + wl.g_offset);
  float* act[2] = {reinterpret_cast<float*>(ws + wl.act_offset), reinterpret_cast<float*>(ws + wl.act_offset + wl.act_stride)};
  hipLaunchKernelGGL(lstm_init_kernel, sg, sb, 0, st, h_init, hstate[0], nstate);

  bool vec = d % 4 == 0 && al16(x) && al16(workspace);
  for (int l = 0; l < n_layers && vec; ++l) vec = al16(W[l]) && al16(U[l]);
  const int nw = lstm_step_waves(d);
  const int step_groups = (d + nw - 1) / nw;
  const dim3 step_grid(step_groups < 8192 ? step_groups : 8192), step_block(nw * 64);

  for (long t0 = 0; t0 < L; t0 += block) {
    const int nt = static_cast<int>(L - t0 < block ? L - t0 : block);
    for (int l = 0; l < n_layers; ++l) {
      const float* xin = l == 0 ? x + t0 * d : act[(l - 1) & 1];
      float* out = l == n_layers - 1 ? h + t0 * d : act[l & 1];
      const float* b = (bias && bias[l]) ? bias[l] : nullptr;
      // the part of Eq. 1 without feedback, for the nt steps of the block: one pass over W
      const int rc = vec ? launch_input<true>(W[l], b, xin, d, G, nt, d, st) : launch_input<false>(W[l], b, xin, d, G, nt, d, st);
      if (rc != SSRNN_OK) return rc;
      // the part with feedback: one pass over U per step
      for (int t = 0; t < nt; ++t) {
        const long tg = t0 + t;
        const float* hp = hstate[tg & 1] + static_cast<long>(l) * d;
        float* hn = hstate[(tg + 1) & 1] + static_cast<long>(l) * d;
        float* cl = c_final + static_cast<long>(l) * d;
        if (vec) hipLaunchKernelGGL((lstm_step_kernel<true>), step_grid, step_block, 0, st, U[l], G + static_cast<long>(t) * 4 * d, hp, hn, out + static_cast<long>(t) * d, cl, d);
        else hipLaunchKernelGGL((lstm_step_kernel<false>), step_grid, step_block, 0, st, U[l], G + static_cast<long>(t) * 4 * d, hp, hn, out + static_cast<long>(t) * d, cl, d);
      }
    }
  }
  hipLaunchKernelGGL(lstm_init_kernel, sg, sb, 0, st, hstate[L & 1], h_final, nstate);
  HIP_TRY(hipGetLastError());
  return SSRNN_OK;
}

}  // namespace ssrnn
