// Host-side builder of the static groups that accompany MoGA (Section 3.2 of the paper,
// "Spatial-Temporal Group Attention"): fixed spatial windows x runs of frames inside a shot, with
// the keys of a group extended by frames of the adjacent shots.  The lists depend only on the
// geometry of the latent video and its shot boundaries, so they are built once on the host
// (plain loops, O(N)) and uploaded by the caller; nothing here touches the GPU.
#include <algorithm>
#include <vector>

#include "moga_common.h"

namespace {

struct Geometry {
  int T, Hh, Ww, wh, ww, tg, a_prev, a_next;
  int nwy, nwx;
  std::vector<int> run_first, run_last, run_shot;   // frame range [first, last] and shot position of a run
  std::vector<int> shot_first, shot_last;           // frame range of a shot position
};

int make_geometry(int T, int Hh, int Ww, int wh, int ww, int tg, const int32_t* shot_of_frame,
                  int a_prev, int a_next, Geometry& g) {
  if (T < 1 || Hh < 1 || Ww < 1 || wh < 1 || ww < 1 || tg < 1 || a_prev < 0 || a_next < 0 || !shot_of_frame)
    return MOGA_ERR_INVALID_ARG;
  if ((int64_t)T * Hh * Ww >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  for (int t = 1; t < T; ++t)
    if (shot_of_frame[t] < shot_of_frame[t - 1]) return MOGA_ERR_INVALID_ARG;   // shots are consecutive frames
  g = Geometry{T, Hh, Ww, wh, ww, tg, a_prev, a_next, (Hh + wh - 1) / wh, (Ww + ww - 1) / ww, {}, {}, {}, {}, {}};
  for (int t = 0; t < T; ++t) {
    const bool new_shot = t == 0 || shot_of_frame[t] != shot_of_frame[t - 1];
    if (new_shot) {
      g.shot_first.push_back(t);
      g.shot_last.push_back(t);
    } else {
      g.shot_last.back() = t;
    }
    if (new_shot || t - g.run_first.back() == tg) {
      g.run_first.push_back(t);
      g.run_last.push_back(t);
      g.run_shot.push_back((int)g.shot_first.size() - 1);
    } else {
      g.run_last.back() = t;
    }
  }
  return MOGA_OK;
}

// Calls f(token) for the tokens of window (wy, wx) in frames [f0, f1], ascending.
template <typename F>
void for_window_tokens(const Geometry& g, int f0, int f1, int wy, int wx, F f) {
  const int y1 = std::min(g.Hh, (wy + 1) * g.wh), x1 = std::min(g.Ww, (wx + 1) * g.ww);
  for (int t = f0; t <= f1; ++t)
    for (int y = wy * g.wh; y < y1; ++y)
      for (int x = wx * g.ww; x < x1; ++x) f((int32_t)(((int64_t)t * g.Hh + y) * g.Ww + x));
}

// Frames added to the keys of a run: the last a_prev frames of the previous shot, the first a_next
// frames of the next shot.  Calls f(first_frame, last_frame) for each non-empty range, ascending.
template <typename F>
void for_added_frames(const Geometry& g, int run, F f) {
  const int p = g.run_shot[run];
  if (p > 0 && g.a_prev > 0) f(std::max(g.shot_first[p - 1], g.shot_last[p - 1] - g.a_prev + 1), g.shot_last[p - 1]);
  if (p + 1 < (int)g.shot_first.size() && g.a_next > 0)
    f(g.shot_first[p + 1], std::min(g.shot_last[p + 1], g.shot_first[p + 1] + g.a_next - 1));
}

}  // namespace

extern "C" int moga_stga_index_sizes(int T, int Hh, int Ww, int wh, int ww, int tg,
                                     const int32_t* shot_of_frame, int a_prev, int a_next,
                                     int64_t* n_groups, int64_t* n_keys) {
  Geometry g;
  const int st = make_geometry(T, Hh, Ww, wh, ww, tg, shot_of_frame, a_prev, a_next, g);
  if (st != MOGA_OK) return st;
  if (!n_groups || !n_keys) return MOGA_ERR_INVALID_ARG;
  int64_t nk = 0;
  for (size_t r = 0; r < g.run_first.size(); ++r)
    for (int wy = 0; wy < g.nwy; ++wy)
      for (int wx = 0; wx < g.nwx; ++wx) {
        const int64_t per_frame = (int64_t)(std::min(Hh, (wy + 1) * wh) - wy * wh) * (std::min(Ww, (wx + 1) * ww) - wx * ww);
        int64_t frames = g.run_last[r] - g.run_first[r] + 1;
        for_added_frames(g, (int)r, [&](int f0, int f1) { frames += f1 - f0 + 1; });
        nk += frames * per_frame;
      }
  *n_groups = (int64_t)g.run_first.size() * g.nwy * g.nwx;
  *n_keys = nk;
  if (*n_groups > MOGA_MAX_SEGMENTS || nk >= ((int64_t)1 << 31)) return MOGA_ERR_UNSUPPORTED;
  return MOGA_OK;
}

extern "C" int moga_stga_build_index(int T, int Hh, int Ww, int wh, int ww, int tg,
                                     const int32_t* shot_of_frame, int a_prev, int a_next,
                                     int32_t* q_index, int32_t* q_slot, int32_t* cu_q,
                                     int32_t* kv_index, int32_t* cu_k, int32_t* inv_cu,
                                     int32_t* inv_slots) {
  int64_t G = 0, Nk = 0;
  const int st = moga_stga_index_sizes(T, Hh, Ww, wh, ww, tg, shot_of_frame, a_prev, a_next, &G, &Nk);
  if (st != MOGA_OK) return st;
  if (!q_index || !q_slot || !cu_q || !kv_index || !cu_k || !inv_cu || !inv_slots) return MOGA_ERR_INVALID_ARG;
  Geometry g;
  make_geometry(T, Hh, Ww, wh, ww, tg, shot_of_frame, a_prev, a_next, g);
  const int64_t N = (int64_t)T * Hh * Ww;
  int64_t nq = 0, nk = 0, grp = 0;
  cu_q[0] = 0;
  cu_k[0] = 0;
  for (size_t r = 0; r < g.run_first.size(); ++r)
    for (int wy = 0; wy < g.nwy; ++wy)
      for (int wx = 0; wx < g.nwx; ++wx) {
        for_window_tokens(g, g.run_first[r], g.run_last[r], wy, wx, [&](int32_t tok) {
          q_slot[tok] = (int32_t)nq;
          q_index[nq++] = tok;
          kv_index[nk++] = tok;
        });
        for_added_frames(g, (int)r, [&](int f0, int f1) {
          for_window_tokens(g, f0, f1, wy, wx, [&](int32_t tok) { kv_index[nk++] = tok; });
        });
        ++grp;
        cu_q[grp] = (int32_t)nq;
        cu_k[grp] = (int32_t)nk;
      }
  // for every token, the key slots that list it, ascending
  for (int64_t i = 0; i <= N; ++i) inv_cu[i] = 0;
  for (int64_t j = 0; j < Nk; ++j) ++inv_cu[kv_index[j] + 1];
  for (int64_t i = 0; i < N; ++i) inv_cu[i + 1] += inv_cu[i];
  std::vector<int32_t> fill(inv_cu, inv_cu + N);
  for (int64_t j = 0; j < Nk; ++j) inv_slots[fill[kv_index[j]]++] = (int32_t)j;
  return MOGA_OK;
}
