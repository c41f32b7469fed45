// C boundary of the population update engine: argument checking, workspace
// layout, and the per-step launch schedule.  See include/pop.h for the contract.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/pop.h"
#include "launch.h"

using namespace pop;

// Scratch of pop_act_explore_noalloc: the per-agent noise scales of the call in flight.  One array per GPU for the
// life of the process (1 KiB); host code reaches it only through the address hipGetSymbolAddress returns for the
// device that is current (scratch_address below), never through this name.
constexpr int kStaticMaxP = 256;
static __device__ __align__(256) float scratch[kStaticMaxP];

namespace {

struct SigmaArgs { float s[kStaticMaxP]; };            // travels to the device as a kernel argument (1 KiB)

__global__ void k_stage_sigma(float* dst, SigmaArgs a, int P) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < P) dst[i] = a.s[i];
}

constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices];                     // address of `scratch` on each device, once looked up
std::mutex g_scratch_mutex;

// Address of the static scratch array on the device that is current (looked up once per device).
hipError_t scratch_address(float** out, int* device) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  *device = dev;
  return hipSuccess;
}

constexpr int64_t kAlign = 256;
constexpr int64_t kStagingBytes = 16ll << 20;

struct Layout {
  int64_t hp, theta, target, m, v, grad, count, cursor, idx, batch, atilde, api, y;
  int64_t cH1, cdZ2, cdZ1, aH1, aH2, adZ2, adZ1, cpart, apart, losses, y_tagged, done_c, done_wc, done_a, spart, sloss, sigma, log_alpha, staging, replay, total;
  int64_t param_bytes;
};

int64_t up(int64_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

thread_local std::string g_create_error;

}  // namespace

struct pop_ctx {
  pop_config cfg;
  PopDev d;
  Layout lay;
  char* ws;
  hipStream_t stream;
  std::vector<pop_hparams> hp;
  std::vector<HpDev> hp_dev;
  std::vector<uint64_t> count;   // host mirror of the buffer fill levels
  uint64_t t;                    // update steps taken
  uint64_t gathered_t;           // step whose batch already sits in its half of the double buffer
  uint32_t step_launches;        // launches of the step kernel so far (alternates its hand-over counters)
  bool handover_pending;         // a launch with waits between its workgroups was enqueued since the fault words were last read
  uint32_t* fault_host;          // two words of pinned host memory the kernels mark when a wait runs out
  float* static_scratch;         // this device's copy of the static scratch array (pop_act_explore_noalloc)
  int device;                    // the device that was current at pop_create
  int fuse;                      // launch structure of a step, see POP_K_* in pop.h: 0 one launch per part, 1 target and
                                 // critic chains in one launch, 2 one launch per step, 3 as 1 plus the rest of a
                                 // delayed step in one launch
  std::string err;
};

namespace {

int fail(pop_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf; else g_create_error = buf;
  return code;
}

#define HIP_TRY(ctx, call)                                                                     \
  do {                                                                                         \
    hipError_t e_ = (call);                                                                    \
    if (e_ != hipSuccess) return fail(ctx, POP_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

// Call after the stream has been synchronised: a wait between workgroups that ran out (chains.h) left marks in
// the two fault words, which live in pinned host memory the device writes to directly (so this costs no copy).
// Reported once, then cleared, so that the context can be used again after its state is restored.
int check_fault(pop_ctx* ctx) {
  if (!ctx->handover_pending) return POP_OK;
  ctx->handover_pending = false;
  volatile uint32_t* f = ctx->fault_host;
  const uint32_t fault = (f[0] ? 1u : 0u) | (f[1] ? 2u : 0u);
  if (!fault) return POP_OK;
  f[0] = 0u; f[1] = 0u;
  return fail(ctx, POP_EHIP, "a wait between workgroups of a fused launch ran into its time limit (fault bits %u: 1 = Bellman targets, "
              "2 = a hand-over count): the results of that step and every later one are invalid", fault);
}

int check_config(const pop_config* c, pop_ctx* ctx) {
  if (!c) return fail(ctx, POP_EINVAL, "config is NULL");
  if (c->P < 1 || c->obs_dim < 1 || c->act_dim < 1 || c->batch < 1 || c->capacity < 1 || c->n_hidden < 1 ||
      c->n_hidden > 4)
    return fail(ctx, POP_EINVAL, "config has a non-positive size");
  if (c->algo != POP_ALGO_TD3 && c->algo != POP_ALGO_SAC && c->algo != POP_ALGO_TD3_SHARED)
    return fail(ctx, POP_EINVAL, "unknown algorithm %d", c->algo);
  if (c->n_hidden != 2 || c->hidden[0] != kH || c->hidden[1] != kH)
    return fail(ctx, POP_EUNSUPPORTED, "hidden layers must be {256, 256}");
  // first-layer fan-in: the chains with a pipelined first layer go up to kSacMaxIn, their wide scratch rows up to
  // kSacMaxAct actions
  const int max_in = kSacMaxIn, max_act = kSacMaxAct;
  if (c->obs_dim + c->act_dim > max_in) return fail(ctx, POP_EUNSUPPORTED, "obs_dim + act_dim must be <= %d", max_in);
  if (c->act_dim > max_act) return fail(ctx, POP_EUNSUPPORTED, "act_dim must be <= %d", max_act);
  if (c->batch != 256) return fail(ctx, POP_EUNSUPPORTED, "batch must be 256");
  if (c->capacity > 0xFFFFFFFFll) return fail(ctx, POP_EUNSUPPORTED, "capacity must be below 2^32");
  if ((int64_t)c->P * c->batch > (1ll << 24)) return fail(ctx, POP_EUNSUPPORTED, "P * batch too large");
  const pop_tuning& u = c->tuning;
  auto rows_ok = [](int r, bool chain16) { return r == 0 || r == 32 || r == 64 || (chain16 && r == 16); };
  if (u.launch < POP_LAUNCH_AUTO || u.launch > POP_LAUNCH_TAIL) return fail(ctx, POP_EINVAL, "tuning.launch %d is not a POP_LAUNCH_* value", u.launch);
  if (!rows_ok(u.rows_target, true) || !rows_ok(u.rows_critic, false) || !rows_ok(u.rows_actor, true))
    return fail(ctx, POP_EINVAL, "tuning.rows_*: 0, 32 or 64 (16 as well for the target and actor chains)");
  if (u.rows_critic1 != 0 && u.rows_critic1 != 16 && u.rows_critic1 != u.rows_critic)
    return fail(ctx, POP_EINVAL, "tuning.rows_critic1: 0, 16 or the value of rows_critic");
  if (u.half_tiles < 0 || u.half_tiles > 2) return fail(ctx, POP_EINVAL, "tuning.half_tiles: 0 (choose), 1 (off) or 2 (on)");
  if (u.actor_ahead < 0 || u.actor_ahead > 2) return fail(ctx, POP_EINVAL, "tuning.actor_ahead: 0 (choose), 1 (off) or 2 (on)");
  return POP_OK;
}

void fill_dims(const pop_config& c, PopDev& d) {
  std::memset(&d, 0, sizeof d);
  d.algo = c.algo;
  d.P = c.P; d.O = c.obs_dim; d.A = c.act_dim; d.D = c.obs_dim + c.act_dim; d.B = c.batch;
  d.row = 2 * c.obs_dim + c.act_dim + 2;
  // Rows per workgroup of the layer chains.  16 for the target and actor chains of small
  // populations: those parts have only 8 P workgroups at 32 rows, well under the 256 CUs, and
  // their latency is what a step waits for; 16-row tiles halve the matrix time of every
  // product by spreading it over twice the CUs.  Else 32.  (64-row chains for all three parts, half the weight
  // traffic per row, exist as well -- tuning.rows_* = 64 -- and were the choice from 128 agents on until the 32-row
  // products learnt to issue their loads between the MFMAs: 1297 against 1278 us/step at P = 256, equal at 128.)
  const int cls = (int64_t)c.P * (c.batch / 16) <= kCUs ? 0 : 1;   // 16-row chains of a part get a CU each
  d.rows_t = d.rows_a = cls == 0 ? 16 : 32;
  // Beside 16 P target workgroups of 16 rows, 64-row critic chains (8 P workgroups) keep the fused
  // target/critic launch of a small population within one workgroup per CU.
  d.rows_c = cls == 1 ? 32 : 64;
  // Small class: 32-row critic chains (16 P workgroups) where they still fit one round of one workgroup
  // per CU beside the target chains (P <= 8) -- the critics' backward pass, which starts when the targets arrive, is
  // the tail of that launch and halves: 81 against 91 us/step at P = 8 -- and from 11 agents on, where neither class
  // fits one round beside the targets and the two chains are launches of their own (98 against 111 us/step at
  // P = 12, 108 against 126 at P = 16).  In between (P = 9, 10: 24 P <= 256 < 32 P) the 64-row class stays.  Shared
  // critics measure alike (98 -> 89 us/step at P = 8, 122 -> 109 at P = 12); SAC, whose steps are longer, gains
  // from the 32-row critic chains throughout (177 -> 157 us/step at P = 10 as launches of their own).
  const int64_t b16 = (int64_t)c.P * (c.batch / 16);
  if (cls == 0 && (c.algo == POP_ALGO_SAC || 2 * b16 <= kCUs || b16 + b16 / 2 > kCUs)) d.rows_c = 32;
  // 9 and 10 agents (24 P <= 256 < 32 P), TD3 proper, target and critic chains in one launch: the 16-row target
  // workgroups go on into critic 1 for their own rows (no hand-over, nothing waits), and only critic 2 has
  // workgroups of its own, 32 rows each: 16 P + 8 P workgroups as before, but the tail after the targets is a
  // 16-row critic chain or a 32-row backward pass instead of a 64-row backward pass (88 against 92 us/step at P = 10).
  d.rows_c1 = 0;
  const pop_tuning& u = c.tuning;
  if (c.algo == POP_ALGO_TD3 && cls == 0 && (u.launch == POP_LAUNCH_AUTO || u.launch == POP_LAUNCH_TARGET_CRITIC)) {
    if (d.rows_c == 64) { d.rows_c = 32; d.rows_c1 = 16; }
    // 11 and 12 agents (20 P <= 256 < 24 P): the same with 64-row workgroups for critic 2 -- 93 against 98 us/step
    else if (b16 + b16 / 2 > kCUs && b16 + b16 / 4 <= kCUs) { d.rows_c = 64; d.rows_c1 = 16; }
  }
  if (c.algo == POP_ALGO_SAC && cls == 1) {           // one launch per chain, so each takes the rows that suit it:
    // 64-row critic chains while they still fit one round of one workgroup per CU (51 against 59 us at P = 32),
    // 16-row target chains while they fit one round of two per CU (44 against 46 us); the actor chain stays at 32
    if ((int64_t)c.P * (c.batch / 64) * 2 <= kCUs) d.rows_c = 64;
    if ((int64_t)c.P * (c.batch / 16) <= 2 * kCUs) d.rows_t = 16;
  }
  // the caller's choices (measurements, tests); naming any chain's rows drops the critic-1 class unless it is named too
  if (u.rows_target || u.rows_critic || u.rows_actor || u.rows_critic1) {
    if (u.rows_target) d.rows_t = u.rows_target;
    if (u.rows_critic) d.rows_c = u.rows_critic;
    if (u.rows_actor) d.rows_a = u.rows_actor;
    d.rows_c1 = u.rows_critic1 == 16 ? 16 : 0;
  }
  // Wide inputs or (TD3) actions (kernels with a pipelined first layer): 32-row chains -- with weights of
  // 2 MB per agent, 16-row workgroups re-read them from L2 often enough to be bound by that -- except
  // for populations too small to fill the chip with them.
  if (d.D > kMaxIn || (c.algo != POP_ALGO_SAC && d.A > kMaxAct)) { d.rows_t = d.rows_a = (int64_t)c.P * (c.batch / 16) <= kCUs ? 16 : 32; d.rows_c = 32; d.rows_c1 = 0; }
  if (d.rows_c1 == 0) d.rows_c1 = d.rows_c;
  d.cstride = d.B / (d.rows_c1 < d.rows_c ? d.rows_c1 : d.rows_c);
  // Stand-alone weight-gradient launches: with fewer than two 32 x 128 tiles per CU (19 workgroups per network at
  // these shapes) some CUs hold two tiles and others one, and the launch lasts as long as the former; tiles of
  // half the width (37 workgroups per network) spread evenly while all of them are resident at three per CU, i.e.
  // up to 10 agents: 73 -> 69 us/step at P = 2, 81 -> 79 at P = 8, 87.8 -> 85.6 at P = 10 (93.5 -> 94.3 at P = 12).
  // The sums over the batch then come in two halves, so comparisons of launch structures bit for bit switch them off.
  d.half_tiles = u.half_tiles ? u.half_tiles == 2 : 2 * (int64_t)c.P * 37 <= 3 * kCUs;
  d.actor = make_layout(d.O, c.algo == POP_ALGO_SAC ? 2 * d.A : d.A);   // SAC: mean and log-std per action
  d.critic = make_layout(d.D, 1);
  d.agent_sz = d.actor.padded + 2 * d.critic.padded;
  d.capacity = (uint64_t)c.capacity;
  d.actor_ahead = 0;                                   // pop_create decides, once the launch structure is known
  d.share = 1;
  if (c.algo == POP_ALGO_TD3_SHARED) {
    // groups of agents whose critic gradients are summed by separate workgroups: as many as keep the partial
    // launch (2 networks x groups x roles workgroups) within the 768 the chip holds at once (three per CU)
    const int roles = 16 + 2 * ((d.critic.in + 31) / 32) + 1;
    d.share = c.P;
    d.groups = std::max(1, std::min(c.P, 3 * kCUs / (2 * roles)));
  }
}

// The chains size their LDS from the shapes: refuse what one CU cannot hold.
int check_fit(const PopDev& d, pop_ctx* ctx) {
  const size_t need = d.algo == POP_ALGO_SAC ? sac_lds_bytes(d) : td3_lds_bytes(d);
  if (need > kLdsPerCU)
    return fail(ctx, POP_EUNSUPPORTED, "obs_dim %d, act_dim %d need %zu bytes of LDS per workgroup, %d available", d.O, d.A,
                need, kLdsPerCU);
  return POP_OK;
}

Layout make_ws_layout(const PopDev& d) {
  Layout L;
  int64_t o = 0;
  auto take = [&](int64_t bytes) { int64_t at = o; o += up(bytes); return at; };
  const int64_t P = d.P, B = d.B;
  L.param_bytes = P * (int64_t)d.agent_sz * 4;
  L.hp = take(P * (int64_t)sizeof(HpDev));
  L.theta = take(L.param_bytes); L.target = take(L.param_bytes);
  L.m = take(L.param_bytes); L.v = take(L.param_bytes); L.grad = take(L.param_bytes);
  L.count = take(P * 4); L.cursor = take(P * 4);
  L.idx = take(2 * P * B * 4); L.batch = take(2 * P * B * d.row * 4);
  L.atilde = take(P * B * d.A * 4); L.api = take(P * B * d.A * 4); L.y = take(P * B * 4);
  const int64_t act = P * B * kH * 4;
  L.cH1 = take(2 * act); L.cdZ2 = take(2 * act); L.cdZ1 = take(2 * act);
  L.aH1 = take(act); L.aH2 = take(act); L.adZ2 = take(act); L.adZ1 = take(act);
  L.cpart = take(P * 2 * (int64_t)d.cstride * kCPart * 4);
  L.apart = take(P * (int64_t)(d.B / d.rows_a) * kAPart * 4);
  L.losses = take(P * 4 * 4);
  L.y_tagged = take(P * B * 8);
  L.done_c = take(4 * P * 4); L.done_wc = take(4 * P * 4); L.done_a = take(2 * P * 4);
  L.spart = take(2 * (int64_t)d.groups * d.critic.padded * 4);
  L.sloss = take(2 * (int64_t)d.groups * 4);
  L.sigma = take(P * 4);
  L.log_alpha = take(3 * P * 4);
  L.staging = take(kStagingBytes);
  L.replay = take(P * (int64_t)d.capacity * d.row * 4);
  L.total = o;
  return L;
}

uint64_t mix64(uint64_t seed, uint64_t i) {   // splitmix64 finaliser of seed + (i + 1) * golden ratio
  uint64_t z = seed + (i + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z ? z : 1;
}

float glorot_limit(int fan_in, int fan_out) { return sqrtf(6.0f / (float)(fan_in + fan_out)); }

const NetLayout* net_of(const PopDev& d, int which, int* net, int64_t* base_off_bytes, const Layout& L,
                        int64_t* region) {
  // which in [0, 15): region = which / 3 for theta, target, m, v, grad in that order
  static const int order[5] = {0, 1, 2, 3, 4};
  const int reg = order[which / 3];
  *net = which % 3;
  const int64_t regs[5] = {L.theta, L.target, L.m, L.v, L.grad};
  *region = regs[reg];
  int64_t off = 0;
  if (*net >= 1) off += d.actor.padded;
  if (*net >= 2) off += d.critic.padded;
  *base_off_bytes = off * 4;
  return *net == 0 ? &d.actor : &d.critic;
}

}  // namespace

extern "C" {

int64_t pop_workspace_bytes(const pop_config* cfg) {
  int rc = check_config(cfg, nullptr);
  if (rc != POP_OK) return rc;
  PopDev d;
  fill_dims(*cfg, d);
  if ((rc = check_fit(d, nullptr)) != POP_OK) return rc;
  return make_ws_layout(d).total;
}

int64_t pop_net_size(const pop_config* cfg, int32_t which) {
  int rc = check_config(cfg, nullptr);
  if (rc != POP_OK) return rc;
  if (which >= POP_LOG_ALPHA && which <= POP_ADAM_V_LOG_ALPHA) return 1;
  if (which < 0 || which > POP_GRAD_CRITIC2) return fail(nullptr, POP_EINVAL, "bad tensor code %d", which);
  PopDev d;
  fill_dims(*cfg, d);
  return which % 3 == 0 ? d.actor.size : d.critic.size;
}

namespace {
int check_hparams(pop_ctx* ctx, const pop_hparams& h, int i) {
  if (h.policy_delay < 1) return fail(ctx, POP_EINVAL, "agent %d: policy_delay must be >= 1", i);
  if (!(h.adam_b1 >= 0.f && h.adam_b1 < 1.f && h.adam_b2 >= 0.f && h.adam_b2 < 1.f && h.adam_eps > 0.f))
    return fail(ctx, POP_EINVAL, "agent %d: Adam constants out of range", i);
  if (!(h.noise_clip >= 0.f) || !(h.policy_noise >= 0.f) || !(h.tau >= 0.f && h.tau <= 1.f))
    return fail(ctx, POP_EINVAL, "agent %d: noise or tau out of range", i);
  return POP_OK;
}

// device copy of one agent's hyperparameters; actor_base / t_base are left to the caller
void to_device_hp(const pop_hparams& h, HpDev& g) {
  g.seed_lo = (uint32_t)h.seed; g.seed_hi = (uint32_t)(h.seed >> 32);
  g.lr_actor = h.lr_actor; g.lr_critic = h.lr_critic; g.gamma = h.gamma; g.tau = h.tau;
  g.policy_noise = h.policy_noise; g.noise_clip = h.noise_clip; g.policy_delay = h.policy_delay;
  g.b1 = h.adam_b1; g.b2 = h.adam_b2; g.eps = h.adam_eps;
  g.lr_alpha = h.lr_alpha; g.target_entropy = h.target_entropy;
}

// actor updates of agent a taken in steps [0, t_now): those before t_base plus the multiples of its delay since
uint32_t actor_updates_before(const pop_ctx* ctx, int a, uint64_t t_now);
}  // namespace

int pop_create(pop_ctx** out, const pop_config* cfg, const pop_hparams* hp, uint64_t seed, void* workspace,
               int64_t workspace_bytes, void* hip_stream) {
  if (!out) return fail(nullptr, POP_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = check_config(cfg, nullptr);
  if (rc != POP_OK) return rc;
  if (!hp) return fail(nullptr, POP_EINVAL, "hp is NULL");
  if (!workspace) return fail(nullptr, POP_EINVAL, "workspace is NULL");
  if (((uintptr_t)workspace % kAlign) != 0) return fail(nullptr, POP_EINVAL, "workspace must be 256-byte aligned");
  for (int i = 0; i < cfg->P; ++i)
    if ((rc = check_hparams(nullptr, hp[i], i)) != POP_OK) return rc;
  if (cfg->algo == POP_ALGO_TD3_SHARED)
    for (int i = 1; i < cfg->P; ++i)
      if (hp[i].policy_delay != hp[0].policy_delay)
        return fail(nullptr, POP_EINVAL, "shared critics: agent %d has policy_delay %d, agent 0 has %d", i, hp[i].policy_delay, hp[0].policy_delay);
  PopDev d;
  fill_dims(*cfg, d);
  if ((rc = check_fit(d, nullptr)) != POP_OK) return rc;
  const Layout L = make_ws_layout(d);
  if (workspace_bytes < L.total)
    return fail(nullptr, POP_ENOMEM, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes,
                (long long)L.total);

  pop_ctx* ctx = new pop_ctx();
  ctx->cfg = *cfg;
  ctx->lay = L;
  ctx->ws = (char*)workspace;
  ctx->stream = (hipStream_t)hip_stream;
  ctx->t = 0;
  ctx->gathered_t = ~0ull;
  ctx->step_launches = 0;
  ctx->handover_pending = false;
  // One launch per step (parts handing over between workgroups), target and critic chains in one launch and the
  // rest in launches of their own, or one launch per part -- by measurement over P = 2 .. 128 (us/step, 64-row
  // critic chains up to P = 16; single launch / target+critic fused / per part): 78 / 83 / - at P = 2, 84 / 85 / -
  // at P = 5, 92 / 91 / - at P = 8, 94.5 / 92.6 / - at P = 10, 111 / 115 / 116 at P = 12, 138 / 126 / 127 at P = 16,
  // 159 / 134 / 158 at P = 20, 185 / 166 / 177 at P = 32, 197 / 210 / 259 at P = 36, 251 / 257 / - at P = 48,
  // 323 / 315 / - at P = 64, 402 / 403 / - at P = 80, 486 / 464 / - at P = 96, 650 / 616 / - at P = 128; with 32-row
  // critic chains beside 16-row target chains, target+critic fused / per part: 73 / 88 at P = 2, 75 / 90 at P = 6,
  // 81 / 96 at P = 8, 101 / 97 at P = 10, - / 98 at P = 12, - / 108 at P = 16, - / 161 at P = 18.
  // Up to 12 agents: target and critic chains fit the chip at once, one workgroup per CU (from 9 agents on with
  // critic 1 inside the target workgroups: fill_dims), and the stand-alone tile kernel holds all the tiles at three
  // per CU where the single launch, one workgroup per CU, needs a second round for them.  13 .. 16: the chains no
  // longer fit at once; each as a launch of its own fills the chip with one round of 16-row (target, actor) or
  // 32-row (critic) workgroups.  17 .. 33: target and critic chains share a
  // launch, two workgroups per CU; waiting weight-gradient workgroups would take the slots the actor chains could
  // start in.  From P = 34 the parts are each several times larger than the 512 workgroups the chip holds and the
  // tails of one part overlap the next inside a single launch; towards a hundred agents the separate launches are
  // ahead again (their tile kernel runs three workgroups per CU, the tiles inside the single launch two).
  const int64_t tc_blocks = (int64_t)cfg->P * (cfg->batch / d.rows_t) + (int64_t)cfg->P * (cfg->batch / d.rows_c) +
                            (d.rows_c1 == d.rows_c ? (int64_t)cfg->P * (cfg->batch / d.rows_c) : 0);
  const int64_t chain_blocks = (int64_t)cfg->P * (cfg->batch / 32) * 3;
  const bool large = d.rows_t == 32 && d.rows_c == 32 && chain_blocks > 800 && chain_blocks <= 2000;   // 34 <= P <= 83
  ctx->fuse = large ? 2 : 1;
  if (d.rows_t == 16 && d.rows_c == 32 && tc_blocks > kCUs) ctx->fuse = 0;   // 13 <= P <= 16
  // SAC: the target and critic chains share a launch where all their workgroups get a CU each (16-row target and
  // 32-row critic chains up to P = 8: 142 against 157 us/step there); measured at P = 32, fusing them loses 4 %
  if (cfg->algo == POP_ALGO_SAC) ctx->fuse = (d.rows_t == 16 && d.rows_c == 32 && tc_blocks <= kCUs) ? 1 : 0;
  if (cfg->algo == POP_ALGO_TD3_SHARED) ctx->fuse = 1;   // target and critic chains together; the critic's weight step is a reduction of its own
  if (cfg->tuning.launch != POP_LAUNCH_AUTO) ctx->fuse = cfg->tuning.launch - POP_LAUNCH_PER_PART;   // 0 .. 3
  if (d.D > kMaxIn || d.A > kMaxAct) ctx->fuse = 0; // wide inputs or actions: the chains exist as separate launches only
  if (cfg->algo == POP_ALGO_TD3_SHARED && ctx->fuse > 1) ctx->fuse = 1;
  if (d.rows_c1 != d.rows_c && (ctx->fuse != 1 || cfg->algo != POP_ALGO_TD3 || d.rows_t != 16 || d.rows_c1 != 16)) {
    delete ctx;
    return fail(nullptr, POP_EINVAL, "tuning.rows_critic1 = 16 needs TD3, rows_target = 16 and POP_LAUNCH_TARGET_CRITIC");
  }
  // The actor's forward pass inside the target / critic launch: where the 32-row workgroups of critic 2 stand idle
  // beside 16-row target workgroups (their forward pass takes 12 us, the targets arrive after 27) and every workgroup
  // of the launch has a CU of its own.
  {
    const bool exists = ctx->fuse == 1 && cfg->algo != POP_ALGO_SAC && d.rows_t == 16 && d.rows_c == 32 && d.rows_a == 16 && d.D <= kMaxIn;
    if (cfg->tuning.actor_ahead == 2 && !exists) {
      delete ctx;
      return fail(nullptr, POP_EINVAL, "tuning.actor_ahead = 2 needs TD3 or shared critics, POP_LAUNCH_TARGET_CRITIC and rows (16, 32, 16)");
    }
    // Measured (us/step, off / on): 79.0 / 77.8 at P = 10, 78.1 / 76.6 at P = 9, 73.0 / 73.1 at P = 8, 65.7 / 65.5 at
    // P = 4: the pass takes 17 us in a 32-row workgroup and the wait it fills is 11 us long, so the launch grows by
    // most of what the actor launch saves -- except where the target workgroups, which run critic 1 as well
    // (rows_c1 == 16), are the longer ones anyway.
    d.actor_ahead = cfg->tuning.actor_ahead ? (cfg->tuning.actor_ahead == 2) : (exists && d.rows_c1 == 16 && tc_blocks <= kCUs);
  }
  if (ctx->fuse >= 2 && d.rows_t == 16 && d.rows_c != 64) {   // the single launch exists for the (16, 64, 16) small class only
    delete ctx;
    return fail(nullptr, POP_EINVAL, "POP_LAUNCH_SINGLE and POP_LAUNCH_TAIL need rows (16, 64, 16) for a population this small");
  }
  ctx->hp.assign(hp, hp + cfg->P);
  if (cfg->algo == POP_ALGO_SAC)
    for (auto& h : ctx->hp) h.policy_delay = 1;
  ctx->count.assign(cfg->P, 0);
  ctx->hp_dev.resize(cfg->P);
  for (int i = 0; i < cfg->P; ++i) {
    pop_hparams& h = ctx->hp[i];
    if (h.seed == 0) h.seed = mix64(seed, (uint64_t)i);
    HpDev& g = ctx->hp_dev[i];
    std::memset(&g, 0, sizeof g);                    // actor_base = t_base = 0
    to_device_hp(h, g);
    if (cfg->algo == POP_ALGO_SAC) g.policy_delay = 1;   // SAC updates everything every step
  }
  char* w = ctx->ws;
  d.theta = (float*)(w + L.theta); d.target = (float*)(w + L.target); d.m = (float*)(w + L.m);
  d.v = (float*)(w + L.v); d.grad = (float*)(w + L.grad); d.record_grads = 0;
  d.hp = (const HpDev*)(w + L.hp);
  d.replay = (float*)(w + L.replay);
  d.count = (uint32_t*)(w + L.count); d.cursor = (uint32_t*)(w + L.cursor);
  d.idx = (uint32_t*)(w + L.idx); d.batch = (float*)(w + L.batch);
  d.atilde = (float*)(w + L.atilde); d.api = (float*)(w + L.api); d.y = (float*)(w + L.y);
  d.cH1 = (float*)(w + L.cH1); d.cdZ2 = (float*)(w + L.cdZ2); d.cdZ1 = (float*)(w + L.cdZ1);
  d.aH1 = (float*)(w + L.aH1); d.aH2 = (float*)(w + L.aH2); d.adZ2 = (float*)(w + L.adZ2);
  d.adZ1 = (float*)(w + L.adZ1);
  d.cpart = (float*)(w + L.cpart); d.apart = (float*)(w + L.apart); d.losses = (float*)(w + L.losses);
  d.y_tagged = (uint64_t*)(w + L.y_tagged); d.done_c = (uint32_t*)(w + L.done_c); d.done_wc = (uint32_t*)(w + L.done_wc); d.done_a = (uint32_t*)(w + L.done_a);
  d.fault = nullptr;                                   // set below, once the pinned words exist
  d.wait_limit = 5000000ull;                           // 50 ms
  d.log_alpha = (float*)(w + L.log_alpha);
  d.spart = (float*)(w + L.spart); d.sloss = (float*)(w + L.sloss);
  ctx->d = d;

  ctx->fault_host = nullptr;
  auto bail = [&](hipError_t e, const char* what) {
    rc = fail(nullptr, POP_EHIP, "%s: %s", what, hipGetErrorString(e));
    if (ctx->fault_host) (void)hipHostFree(ctx->fault_host);
    delete ctx;
    return rc;
  };
  hipError_t e;
  if ((e = setup_kernels()) != hipSuccess || (e = setup_step_kernel()) != hipSuccess || (e = setup_sac_kernels()) != hipSuccess)
    return bail(e, "kernel attribute setup");
  if ((e = scratch_address(&ctx->static_scratch, &ctx->device)) != hipSuccess) return bail(e, "hipGetSymbolAddress(scratch)");
  // the two fault words: 8 bytes of pinned host memory, mapped into the device's address space
  void* fh = nullptr;
  if ((e = hipHostMalloc(&fh, 2 * sizeof(uint32_t), hipHostMallocMapped)) != hipSuccess) return bail(e, "hipHostMalloc(fault words)");
  ctx->fault_host = (uint32_t*)fh;
  ctx->fault_host[0] = ctx->fault_host[1] = 0u;
  void* fd = nullptr;
  if ((e = hipHostGetDevicePointer(&fd, fh, 0)) != hipSuccess) { (void)hipHostFree(fh); return bail(e, "hipHostGetDevicePointer"); }
  ctx->d.fault = (uint32_t*)fd;
  hipStream_t s = ctx->stream;
  // everything between the hyperparameters and the staging area starts at zero
  if ((e = hipMemsetAsync(w, 0, (size_t)L.staging, s)) != hipSuccess) return bail(e, "hipMemsetAsync");
  if ((e = hipMemcpyAsync(w + L.hp, ctx->hp_dev.data(), sizeof(HpDev) * cfg->P, hipMemcpyHostToDevice, s)) != hipSuccess)
    return bail(e, "hipMemcpyAsync(hparams)");
  InitLimits lim;
  lim.actor[0] = glorot_limit(d.O, kH); lim.actor[1] = glorot_limit(kH, kH); lim.actor[2] = glorot_limit(kH, d.actor.out);
  lim.critic[0] = glorot_limit(d.D, kH); lim.critic[1] = glorot_limit(kH, kH); lim.critic[2] = glorot_limit(kH, 1);
  if ((e = launch_init(ctx->d, lim, s)) != hipSuccess) return bail(e, "init kernel");
  if (cfg->algo == POP_ALGO_SAC) {                 // log temperature; its Adam moments stay zero
    std::vector<float> la(cfg->P);
    for (int i = 0; i < cfg->P; ++i) la[i] = ctx->hp[i].init_log_alpha;
    if ((e = hipMemcpyAsync(d.log_alpha, la.data(), sizeof(float) * cfg->P, hipMemcpyHostToDevice, s)) != hipSuccess ||
        (e = hipStreamSynchronize(s)) != hipSuccess)
      return bail(e, "hipMemcpyAsync(log_alpha)");
  }
  if ((e = hipStreamSynchronize(s)) != hipSuccess) return bail(e, "hipStreamSynchronize");
  *out = ctx;
  return POP_OK;
}

int pop_insert(pop_ctx* ctx, int32_t agent, int64_t n, const float* obs, const float* act, const float* rew,
               const float* done, const float* next_obs, int32_t ptrs_on_device) {
  if (!ctx) return POP_EINVAL;
  if (agent < -1 || agent >= ctx->d.P) return fail(ctx, POP_EINVAL, "agent %d out of range", agent);
  if (n < 0 || n > 0xFFFFFFFFll) return fail(ctx, POP_EINVAL, "n out of range");
  if (n == 0) return POP_OK;
  if (!obs || !act || !rew || !done || !next_obs) return fail(ctx, POP_EINVAL, "NULL transition array");
  ctx->gathered_t = ~0ull;        // a batch drawn before this insert would not see the new rows
  const PopDev& d = ctx->d;
  hipStream_t s = ctx->stream;
  auto bump = [&](int a, int64_t k) {
    ctx->count[a] = std::min<uint64_t>(ctx->count[a] + (uint64_t)k, d.capacity);
  };
  if (ptrs_on_device) {
    HIP_TRY(ctx, launch_insert(d, agent, n, obs, act, rew, done, next_obs, s));
    if (agent < 0) for (int a = 0; a < d.P; ++a) bump(a, n); else bump(agent, n);
    return POP_OK;
  }
  // host arrays: stage piecewise through the workspace, one agent at a time
  float* st = (float*)(ctx->ws + ctx->lay.staging);
  const int64_t rows_per_piece = kStagingBytes / ((int64_t)d.row * 4);
  const int a_lo = agent < 0 ? 0 : agent, a_hi = agent < 0 ? d.P : agent + 1;
  for (int a = a_lo; a < a_hi; ++a) {
    const int64_t slice = agent < 0 ? (int64_t)a * n : 0;
    for (int64_t off = 0; off < n; off += rows_per_piece) {
      const int64_t k = std::min(rows_per_piece, n - off);
      float* s_obs = st;
      float* s_act = s_obs + k * d.O;
      float* s_rew = s_act + k * d.A;
      float* s_done = s_rew + k;
      float* s_next = s_done + k;
      const int64_t r = slice + off;
      HIP_TRY(ctx, hipMemcpyAsync(s_obs, obs + r * d.O, k * d.O * 4, hipMemcpyHostToDevice, s));
      HIP_TRY(ctx, hipMemcpyAsync(s_act, act + r * d.A, k * d.A * 4, hipMemcpyHostToDevice, s));
      HIP_TRY(ctx, hipMemcpyAsync(s_rew, rew + r, k * 4, hipMemcpyHostToDevice, s));
      HIP_TRY(ctx, hipMemcpyAsync(s_done, done + r, k * 4, hipMemcpyHostToDevice, s));
      HIP_TRY(ctx, hipMemcpyAsync(s_next, next_obs + r * d.O, k * d.O * 4, hipMemcpyHostToDevice, s));
      HIP_TRY(ctx, launch_insert(d, a, k, s_obs, s_act, s_rew, s_done, s_next, s));
      HIP_TRY(ctx, hipStreamSynchronize(s));      // the staging area is reused by the next piece
      bump(a, k);
    }
  }
  return POP_OK;
}

}  // extern "C"

namespace {

// One update step: launches in stream order.  `tick(k, end)` is called before and after
// kernel k.  The critic weight-gradient kernel also draws and gathers the replay rows of the
// step after this one (whether or not that step belongs to the same call), so a stand-alone
// gather runs only when those rows are not there or no longer valid: at the very first step,
// and after an insert, a buffer copy or new hyperparameters (a new seed draws other rows).
template <class Tick>
int enqueue_step(pop_ctx* ctx, Tick tick) {
  const bool has_next = ctx->t + 1 <= 0xFFFFFFFFull;
  const PopDev& d = ctx->d;
  hipStream_t s = ctx->stream;
  const uint32_t t = (uint32_t)ctx->t;
  hipError_t e = hipSuccess;
  auto run = [&](int k, hipError_t (*fn)(const PopDev&, uint32_t, hipStream_t)) {
    tick(k, 0);
    e = fn(d, t, s);
    tick(k, 1);
    return e == hipSuccess;
  };
  if (ctx->gathered_t != ctx->t && !run(POP_K_GATHER, launch_sample_gather))
    return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
  bool any_actor = false;
  for (int a = 0; a < d.P && !any_actor; ++a) any_actor = (t % (uint32_t)ctx->hp[a].policy_delay) == 0;
  if (ctx->fuse != 0) ctx->handover_pending = true;   // every fused launch has waits between its workgroups
  if (d.algo == POP_ALGO_SAC) {                       // critic chain and tiles are the TD3 ones; fuse = 0: one launch
                                                      // per part, else target and critic chains in one launch
    if (ctx->fuse != 0) {
      if (!run(POP_K_TARGET_CRITIC, launch_sac_target_critic)) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    } else if (!run(POP_K_TARGET, launch_sac_target) || !run(POP_K_CRITIC, launch_critic)) {
      return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    }
    tick(POP_K_WGRAD_CRITIC, 0);
    e = launch_wgrad_adam(d, t, 0, has_next ? 1 : 0, s);
    tick(POP_K_WGRAD_CRITIC, 1);
    if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    if (has_next) ctx->gathered_t = ctx->t + 1;
    if (!run(POP_K_ACTOR, launch_sac_actor)) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    tick(POP_K_WGRAD_ACTOR, 0);
    e = launch_wgrad_adam(d, t, 1, 0, s);
    tick(POP_K_WGRAD_ACTOR, 1);
    if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    ctx->t++;
    return POP_OK;
  }
  if (d.algo == POP_ALGO_TD3_SHARED) {                // the TD3 chains on the shared critic blocks; the critics' weight
                                                      // step sums over the population (k_wgrad_shared.hip)
    if (ctx->fuse != 0) {                             // target and critic chains in one launch (y handed over inside it)
      if (!run(POP_K_TARGET_CRITIC, launch_target_critic)) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    } else if (!run(POP_K_TARGET, launch_target) || !run(POP_K_CRITIC, launch_critic)) {
      return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    }
    tick(POP_K_WGRAD_CRITIC, 0);
    e = launch_wgrad_shared(d, t, has_next ? 1 : 0, s);
    tick(POP_K_WGRAD_CRITIC, 1);
    if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    if (has_next) ctx->gathered_t = ctx->t + 1;
    if (any_actor) {
      if (!run(POP_K_ACTOR, launch_actor)) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
      tick(POP_K_WGRAD_ACTOR, 0);
      e = launch_wgrad_adam(d, t, 1, 0, s);
      tick(POP_K_WGRAD_ACTOR, 1);
      if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    }
    ctx->t++;
    return POP_OK;
  }
  if (ctx->fuse == 2) {
    tick(POP_K_STEP, 0);
    e = launch_step(d, t, ctx->step_launches, 1, any_actor ? 1 : 0, has_next ? 1 : 0, s);
    tick(POP_K_STEP, 1);
    if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    ctx->step_launches++;                            // only a launch that ran has cleared the other half of the counters
    if (has_next) ctx->gathered_t = ctx->t + 1;
    ctx->t++;
    return POP_OK;
  }
  if (ctx->fuse == 1 || ctx->fuse == 3) {
    if (!run(POP_K_TARGET_CRITIC, launch_target_critic)) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    if (any_actor && ctx->fuse == 3) {               // the rest of the step in one launch: the actor's own forward pass
      tick(POP_K_STEP_TAIL, 0);                      // runs beside the critic weight gradients
      e = launch_step(d, t, ctx->step_launches, 0, 1, has_next ? 1 : 0, s);
      tick(POP_K_STEP_TAIL, 1);
      if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
      ctx->step_launches++;
      if (has_next) ctx->gathered_t = ctx->t + 1;
      ctx->t++;
      return POP_OK;
    }
  } else if (!run(POP_K_TARGET, launch_target) || !run(POP_K_CRITIC, launch_critic)) {
    return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
  }
  tick(POP_K_WGRAD_CRITIC, 0);
  e = launch_wgrad_adam(d, t, 0, has_next ? 1 : 0, s);
  tick(POP_K_WGRAD_CRITIC, 1);
  if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
  if (has_next) ctx->gathered_t = ctx->t + 1;
  if (any_actor) {
    if (!run(POP_K_ACTOR, launch_actor)) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
    tick(POP_K_WGRAD_ACTOR, 0);
    e = launch_wgrad_adam(d, t, 1, 0, s);
    tick(POP_K_WGRAD_ACTOR, 1);
    if (e != hipSuccess) return fail(ctx, POP_EHIP, "kernel launch: %s", hipGetErrorString(e));
  }
  ctx->t++;
  return POP_OK;
}

int check_update(pop_ctx* ctx, int32_t n_steps) {
  if (n_steps < 0) return fail(ctx, POP_EINVAL, "n_steps is negative");
  for (int a = 0; a < ctx->d.P; ++a)
    if (ctx->count[a] == 0) return fail(ctx, POP_EEMPTY, "agent %d has an empty replay buffer", a);
  if (ctx->t + (uint64_t)n_steps > 0xFFFFFFFFull) return fail(ctx, POP_EINVAL, "step counter would exceed 2^32");
  return POP_OK;
}

}  // namespace

extern "C" {

int pop_update(pop_ctx* ctx, int32_t n_steps) {
  if (!ctx) return POP_EINVAL;
  int rc = check_update(ctx, n_steps);
  if (rc != POP_OK) return rc;
  for (int i = 0; i < n_steps; ++i)
    if ((rc = enqueue_step(ctx, [](int, int) {})) != POP_OK) return rc;
  return POP_OK;
}

int pop_update_timed(pop_ctx* ctx, int32_t n_steps, double* ms, int64_t* launches) {
  if (!ctx) return POP_EINVAL;
  if (!ms || !launches) return fail(ctx, POP_EINVAL, "NULL output array");
  int rc = check_update(ctx, n_steps);
  if (rc != POP_OK) return rc;
  for (int k = 0; k < POP_K_COUNT; ++k) { ms[k] = 0.0; launches[k] = 0; }
  const int kPiece = 64;                         // steps per batch of events
  std::vector<hipEvent_t> ev((size_t)kPiece * POP_K_COUNT * 2, nullptr);
  for (auto& e : ev) HIP_TRY(ctx, hipEventCreate(&e));
  std::vector<char> used((size_t)kPiece * POP_K_COUNT);
  hipStream_t s = ctx->stream;
  for (int done = 0; done < n_steps && rc == POP_OK; done += kPiece) {
    const int steps = std::min(kPiece, n_steps - done);
    std::fill(used.begin(), used.end(), 0);
    hipError_t ee = hipSuccess;
    for (int i = 0; i < steps && rc == POP_OK; ++i) {
      rc = enqueue_step(ctx, [&](int k, int end) {
        const size_t slot = (size_t)i * POP_K_COUNT + k;
        hipError_t r = hipEventRecord(ev[2 * slot + end], s);
        if (r != hipSuccess) ee = r;
        used[slot] = 1;
      });
    }
    hipError_t se = hipStreamSynchronize(s);
    if (rc == POP_OK && (se != hipSuccess || ee != hipSuccess))
      rc = fail(ctx, POP_EHIP, "timed update: %s", hipGetErrorString(se != hipSuccess ? se : ee));
    if (rc == POP_OK) {
      for (size_t slot = 0; slot < (size_t)steps * POP_K_COUNT; ++slot) {
        if (!used[slot]) continue;
        float t_ms = 0.f;
        if (hipEventElapsedTime(&t_ms, ev[2 * slot], ev[2 * slot + 1]) == hipSuccess) {
          ms[slot % POP_K_COUNT] += t_ms;
          launches[slot % POP_K_COUNT] += 1;
        }
      }
    }
  }
  for (auto& e : ev) (void)hipEventDestroy(e);
  if (rc == POP_OK) rc = check_fault(ctx);
  return rc;
}

namespace {
int act_impl(pop_ctx* ctx, const float* obs, int32_t n, float* act_out, int32_t ptrs_on_device, const float* sigma_dev,
             uint32_t step) {
  if (n < 0) return fail(ctx, POP_EINVAL, "n is negative");
  if (n == 0) return POP_OK;
  if (!obs || !act_out) return fail(ctx, POP_EINVAL, "NULL array");
  const PopDev& d = ctx->d;
  if ((int64_t)n * d.A > 0xFFFFFFFFll) return fail(ctx, POP_EINVAL, "n * act_dim exceeds 2^32");
  hipStream_t s = ctx->stream;
  if (ptrs_on_device) {
    HIP_TRY(ctx, launch_act(d, obs, n, act_out, sigma_dev, step, 0u, s));
    return POP_OK;
  }
  float* st = (float*)(ctx->ws + ctx->lay.staging);
  const int64_t per_row = (int64_t)d.P * (d.O + d.A) * 4;
  if (per_row > kStagingBytes) return fail(ctx, POP_EUNSUPPORTED, "host arrays: one row of all agents exceeds the staging area; pass device pointers");
  const int64_t piece = kStagingBytes / per_row;
  for (int64_t off = 0; off < n; off += piece) {
    const int k = (int)std::min<int64_t>(piece, n - off);
    float* s_obs = st;
    float* s_act = st + (int64_t)d.P * k * d.O;
    HIP_TRY(ctx, hipMemcpy2DAsync(s_obs, (size_t)k * d.O * 4, obs + off * d.O, (size_t)n * d.O * 4, (size_t)k * d.O * 4,
                                  d.P, hipMemcpyHostToDevice, s));
    HIP_TRY(ctx, launch_act(d, s_obs, k, s_act, sigma_dev, step, (uint32_t)off, s));
    HIP_TRY(ctx, hipMemcpy2DAsync(act_out + off * d.A, (size_t)n * d.A * 4, s_act, (size_t)k * d.A * 4,
                                  (size_t)k * d.A * 4, d.P, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
  }
  return check_fault(ctx);
}
}  // namespace

int pop_act(pop_ctx* ctx, const float* obs, int32_t n, float* act_out, int32_t ptrs_on_device) {
  if (!ctx) return POP_EINVAL;
  return act_impl(ctx, obs, n, act_out, ptrs_on_device, nullptr, 0u);
}

int pop_act_explore(pop_ctx* ctx, const float* obs, int32_t n, float* act_out, int32_t ptrs_on_device,
                    const float* sigma, uint32_t step) {
  if (!ctx) return POP_EINVAL;
  if (!sigma) return fail(ctx, POP_EINVAL, "sigma is NULL");
  for (int a = 0; a < ctx->d.P; ++a)
    if (!(sigma[a] >= 0.0f)) return fail(ctx, POP_EINVAL, "agent %d: sigma must be >= 0", a);
  float* sigma_dev = (float*)(ctx->ws + ctx->lay.sigma);
  // the staged values must not change under an earlier call still in flight
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  HIP_TRY(ctx, hipMemcpyAsync(sigma_dev, sigma, sizeof(float) * ctx->d.P, hipMemcpyHostToDevice, ctx->stream));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  return act_impl(ctx, obs, n, act_out, ptrs_on_device, sigma_dev, step);
}

int pop_act_explore_noalloc(pop_ctx* ctx, const float* obs, int32_t n, float* act_out, const float* sigma, uint32_t step) {
  if (!ctx) return POP_EINVAL;
  const PopDev& d = ctx->d;
  if (d.P > kStaticMaxP)
    return fail(ctx, POP_EUNSUPPORTED, "a population of %d agents exceeds the %d the static scratch array holds", d.P, kStaticMaxP);
  if (!sigma) return fail(ctx, POP_EINVAL, "sigma is NULL");
  if (n < 0) return fail(ctx, POP_EINVAL, "n is negative");
  if ((int64_t)n * d.A > 0xFFFFFFFFll) return fail(ctx, POP_EINVAL, "n * act_dim exceeds 2^32");
  SigmaArgs args;
  for (int a = 0; a < d.P; ++a) {
    if (!(sigma[a] >= 0.0f)) return fail(ctx, POP_EINVAL, "agent %d: sigma must be >= 0", a);
    args.s[a] = sigma[a];
  }
  if (n == 0) return POP_OK;
  if (!obs || !act_out) return fail(ctx, POP_EINVAL, "NULL array");
  // two launches in stream order and nothing else: the noise scales go into this device's scratch array as a kernel
  // argument, the acting kernel reads them from there
  k_stage_sigma<<<dim3((d.P + 63) / 64), dim3(64), 0, ctx->stream>>>(ctx->static_scratch, args, d.P);
  HIP_TRY(ctx, hipGetLastError());
  HIP_TRY(ctx, launch_act(d, obs, n, act_out, ctx->static_scratch, step, 0u, ctx->stream));
  return POP_OK;
}

int64_t pop_get_params(pop_ctx* ctx, int32_t agent, int32_t which, float* out, int64_t out_len, int32_t on_device) {
  if (!ctx) return POP_EINVAL;
  if (agent < 0 || agent >= ctx->d.P) return fail(ctx, POP_EINVAL, "agent %d out of range", agent);
  if (which >= POP_LOG_ALPHA && which <= POP_ADAM_V_LOG_ALPHA) {       // SAC temperature: one float
    if (ctx->d.algo != POP_ALGO_SAC) return fail(ctx, POP_EINVAL, "tensor code %d exists for SAC only", which);
    if (!out || out_len < 1) return fail(ctx, POP_EINVAL, "out is NULL or too short");
    const float* src = ctx->d.log_alpha + (size_t)(which - POP_LOG_ALPHA) * ctx->d.P + agent;
    HIP_TRY(ctx, hipMemcpyAsync(out, src, 4, on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, ctx->stream));
    if (!on_device) {
      HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
      const int rc = check_fault(ctx);
      if (rc != POP_OK) return rc;
    }
    return 1;
  }
  if (which < 0 || which > POP_GRAD_CRITIC2) return fail(ctx, POP_EINVAL, "bad tensor code %d", which);
  if (!out) return fail(ctx, POP_EINVAL, "out is NULL");
  int net;
  int64_t off, region;
  const NetLayout* L = net_of(ctx->d, which, &net, &off, ctx->lay, &region);
  if (out_len < L->size) return fail(ctx, POP_EINVAL, "out_len %lld < %d", (long long)out_len, L->size);
  if (ctx->d.share > 1 && net >= 1) agent = 0;         // the shared critics live in agent 0's blocks
  const char* src = ctx->ws + region + (int64_t)agent * ctx->d.agent_sz * 4 + off;
  HIP_TRY(ctx, hipMemcpyAsync(out, src, (size_t)L->size * 4, on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost,
                              ctx->stream));
  if (!on_device) {
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    const int rc = check_fault(ctx);
    if (rc != POP_OK) return rc;
  }
  return L->size;
}

int pop_set_params(pop_ctx* ctx, int32_t agent, int32_t which, const float* in, int64_t in_len, int32_t on_device) {
  if (!ctx) return POP_EINVAL;
  if (agent < 0 || agent >= ctx->d.P) return fail(ctx, POP_EINVAL, "agent %d out of range", agent);
  if (which >= POP_LOG_ALPHA && which <= POP_ADAM_V_LOG_ALPHA) {
    if (ctx->d.algo != POP_ALGO_SAC) return fail(ctx, POP_EINVAL, "tensor code %d exists for SAC only", which);
    if (!in || in_len != 1) return fail(ctx, POP_EINVAL, "in is NULL or in_len != 1");
    float* dst = ctx->d.log_alpha + (size_t)(which - POP_LOG_ALPHA) * ctx->d.P + agent;
    HIP_TRY(ctx, hipMemcpyAsync(dst, in, 4, on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, ctx->stream));
    if (!on_device) HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return POP_OK;
  }
  if (which < 0 || which > POP_ADAM_V_CRITIC2) return fail(ctx, POP_EINVAL, "tensor code %d cannot be written", which);
  if (!in) return fail(ctx, POP_EINVAL, "in is NULL");
  int net;
  int64_t off, region;
  const NetLayout* L = net_of(ctx->d, which, &net, &off, ctx->lay, &region);
  if (in_len != L->size) return fail(ctx, POP_EINVAL, "in_len %lld != %d", (long long)in_len, L->size);
  if (ctx->d.share > 1 && net >= 1) agent = 0;
  char* dst = ctx->ws + region + (int64_t)agent * ctx->d.agent_sz * 4 + off;
  HIP_TRY(ctx, hipMemcpyAsync(dst, in, (size_t)L->size * 4, on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                              ctx->stream));
  if (!on_device) HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  return POP_OK;
}

int pop_set_debug(pop_ctx* ctx, int32_t on) {
  if (!ctx) return POP_EINVAL;
  ctx->d.record_grads = on ? 1 : 0;
  return POP_OK;
}

int64_t pop_debug_get(pop_ctx* ctx, int32_t what, void* out, int64_t out_bytes, int32_t on_device) {
  if (!ctx) return POP_EINVAL;
  if (!out) return fail(ctx, POP_EINVAL, "out is NULL");
  const PopDev& d = ctx->d;
  const int64_t PB = (int64_t)d.P * d.B;
  const char* src = nullptr;
  int64_t bytes = 0;
  const int64_t half = ctx->t > 0 ? (int64_t)((ctx->t - 1) & 1) : 0;   // buffer half of the last step
  switch (what) {
    case POP_DBG_INDICES: bytes = PB * 4; src = (const char*)d.idx + half * bytes; break;
    case POP_DBG_BATCH: bytes = PB * d.row * 4; src = (const char*)d.batch + half * bytes; break;
    case POP_DBG_TARGET_ACTION: src = (const char*)d.atilde; bytes = PB * d.A * 4; break;
    case POP_DBG_TARGET_Y: src = (const char*)d.y; bytes = PB * 4; break;
    case POP_DBG_LOSSES: bytes = (int64_t)d.P * 2 * 4; break;
    default: return fail(ctx, POP_EINVAL, "bad debug code %d", what);
  }
  if (out_bytes < bytes) return fail(ctx, POP_EINVAL, "out_bytes %lld < %lld", (long long)out_bytes, (long long)bytes);
  if (what == POP_DBG_LOSSES) {
    if (on_device) return fail(ctx, POP_EINVAL, "losses are returned to host memory only");
    std::vector<float> raw((size_t)d.P * 4);
    HIP_TRY(ctx, hipMemcpyAsync(raw.data(), d.losses, raw.size() * 4, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    float* o = (float*)out;
    for (int a = 0; a < d.P; ++a) { o[2 * a] = raw[4 * a] + raw[4 * a + 1]; o[2 * a + 1] = raw[4 * a + 2]; }
    const int rc = check_fault(ctx);
    return rc != POP_OK ? rc : bytes;
  }
  HIP_TRY(ctx, hipMemcpyAsync(out, src, (size_t)bytes, on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost,
                              ctx->stream));
  if (!on_device) {
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    const int rc = check_fault(ctx);
    if (rc != POP_OK) return rc;
  }
  return bytes;
}

int pop_debug_indices(pop_ctx* ctx, int64_t* out) {
  if (!ctx) return POP_EINVAL;
  if (!out) return fail(ctx, POP_EINVAL, "out is NULL");
  const int64_t PB = (int64_t)ctx->d.P * ctx->d.B;
  std::vector<uint32_t> raw((size_t)PB);
  int64_t rc = pop_debug_get(ctx, POP_DBG_INDICES, raw.data(), PB * 4, 0);
  if (rc < 0) return (int)rc;
  for (int64_t i = 0; i < PB; ++i) out[i] = (int64_t)raw[(size_t)i];
  return POP_OK;
}

int64_t pop_step_count(const pop_ctx* ctx) { return ctx ? (int64_t)ctx->t : POP_EINVAL; }

int64_t pop_buffer_count(const pop_ctx* ctx, int32_t agent) {
  if (!ctx || agent < 0 || agent >= ctx->d.P) return POP_EINVAL;
  return (int64_t)ctx->count[agent];
}

namespace {
uint32_t actor_updates_before(const pop_ctx* ctx, int a, uint64_t t_now) {
  const HpDev& g = ctx->hp_dev[a];
  const uint64_t d = (uint64_t)g.policy_delay, lo = g.t_base;
  if (t_now <= lo) return g.actor_base;
  const uint64_t hi = t_now - 1;                     // multiples of d in [lo, hi]
  return g.actor_base + (uint32_t)(hi / d - (lo + d - 1) / d + 1);
}
}  // namespace

int pop_set_hparams(pop_ctx* ctx, int32_t agent, const pop_hparams* hp) {
  if (!ctx) return POP_EINVAL;
  if (!hp) return fail(ctx, POP_EINVAL, "hp is NULL");
  if (agent < 0 || agent >= ctx->d.P) return fail(ctx, POP_EINVAL, "agent %d out of range", agent);
  const int rc = check_hparams(ctx, *hp, agent);
  if (rc != POP_OK) return rc;
  if (hp->seed == 0) return fail(ctx, POP_EINVAL, "seed 0 (derive from the population seed) is only meaningful at pop_create");
  if (ctx->d.algo == POP_ALGO_TD3_SHARED && ctx->d.P > 1 && hp->policy_delay != ctx->hp[agent == 0 ? 1 : 0].policy_delay)
    return fail(ctx, POP_EINVAL, "shared critics: policy_delay is common to the population (%d)", ctx->hp[agent == 0 ? 1 : 0].policy_delay);
  HpDev& g = ctx->hp_dev[agent];
  g.actor_base = actor_updates_before(ctx, agent, ctx->t);   // under the old delay, up to now
  g.t_base = (uint32_t)ctx->t;
  ctx->gathered_t = ~0ull;                             // rows gathered ahead were drawn under the old seed
  ctx->hp[agent] = *hp;
  to_device_hp(*hp, g);
  if (ctx->d.algo == POP_ALGO_SAC) { ctx->hp[agent].policy_delay = 1; g.policy_delay = 1; }
  // hp_dev lives as long as the context and is only changed here, after a synchronisation
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  HIP_TRY(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.hp + sizeof(HpDev) * agent, &g, sizeof(HpDev), hipMemcpyHostToDevice, ctx->stream));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  return POP_OK;
}

int pop_copy_agent(pop_ctx* ctx, int32_t dst, int32_t src, int32_t with_buffer) {
  if (!ctx) return POP_EINVAL;
  const PopDev& d = ctx->d;
  if (dst < 0 || dst >= d.P || src < 0 || src >= d.P) return fail(ctx, POP_EINVAL, "agent out of range (dst %d, src %d)", dst, src);
  if (dst == src) return POP_OK;
  hipStream_t s = ctx->stream;
  // the actor block comes first in an agent's state; with shared critics that is all an agent owns
  const size_t state = (size_t)(d.share > 1 ? d.actor.padded : d.agent_sz) * sizeof(float);
  for (float* region : {d.theta, d.target, d.m, d.v})
    HIP_TRY(ctx, hipMemcpyAsync(region + (size_t)dst * d.agent_sz, region + (size_t)src * d.agent_sz, state, hipMemcpyDeviceToDevice, s));
  if (d.algo == POP_ALGO_SAC)
    for (int k = 0; k < 3; ++k)
      HIP_TRY(ctx, hipMemcpyAsync(d.log_alpha + (size_t)k * d.P + dst, d.log_alpha + (size_t)k * d.P + src, sizeof(float), hipMemcpyDeviceToDevice, s));
  if (with_buffer) {
    const size_t rows = (size_t)d.capacity * d.row;
    HIP_TRY(ctx, hipMemcpyAsync(d.replay + (size_t)dst * rows, d.replay + (size_t)src * rows, rows * sizeof(float), hipMemcpyDeviceToDevice, s));
    HIP_TRY(ctx, hipMemcpyAsync(d.count + dst, d.count + src, sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
    HIP_TRY(ctx, hipMemcpyAsync(d.cursor + dst, d.cursor + src, sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
    ctx->count[dst] = ctx->count[src];
    if (ctx->gathered_t == ctx->t) ctx->gathered_t = ~0ull;   // rows already gathered for the next step are stale for dst
  }
  // the Adam state came along, so the count of actor updates does too; dst keeps its own delay from here on
  HpDev& g = ctx->hp_dev[dst];
  g.actor_base = actor_updates_before(ctx, src, ctx->t);
  g.t_base = (uint32_t)ctx->t;
  HIP_TRY(ctx, hipStreamSynchronize(s));
  HIP_TRY(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.hp + sizeof(HpDev) * dst, &g, sizeof(HpDev), hipMemcpyHostToDevice, s));
  HIP_TRY(ctx, hipStreamSynchronize(s));
  return POP_OK;
}

int pop_sync(pop_ctx* ctx) {
  if (!ctx) return POP_EINVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  HIP_TRY(ctx, hipGetLastError());
  return check_fault(ctx);
}

int pop_get_tuning(const pop_ctx* ctx, pop_tuning* out) {
  if (!ctx || !out) return POP_EINVAL;
  const PopDev& d = ctx->d;
  out->launch = POP_LAUNCH_PER_PART + ctx->fuse;
  out->rows_target = d.rows_t; out->rows_critic = d.rows_c; out->rows_actor = d.rows_a; out->rows_critic1 = d.rows_c1;
  out->half_tiles = d.half_tiles ? 2 : 1;
  out->actor_ahead = d.actor_ahead ? 2 : 1;
  return POP_OK;
}

int pop_set_option(pop_ctx* ctx, int32_t key, int64_t value) {
  if (!ctx) return POP_EINVAL;
  switch (key) {
    case POP_OPT_WAIT_LIMIT_TICKS:
      if (value < 1 || value > 1000000000ll) return fail(ctx, POP_EINVAL, "wait limit must be 1 .. 10^9 ticks of 10 ns");
      ctx->d.wait_limit = (unsigned long long)value;
      return POP_OK;
    default:
      return fail(ctx, POP_EINVAL, "unknown option %d", key);
  }
}

int pop_destroy(pop_ctx* ctx) {
  if (!ctx) return POP_EINVAL;
  if (ctx->fault_host) (void)hipHostFree(ctx->fault_host);
  delete ctx;
  return POP_OK;
}

const char* pop_last_error(const pop_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
