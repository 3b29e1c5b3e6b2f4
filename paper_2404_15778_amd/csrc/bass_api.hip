// Version and status strings of libbass, and the host-side draft-length heuristic.
#include "bass_common.h"

extern "C" int bass_version(void) { return 212; /* 0.2.12: step plans (bass_attention_plan) drive every attention launch; bass_warp_accept; 768-wavefront launches as 256 workgroups of three */ }

extern "C" const char* bass_status_string(int code) {
  switch (code) {
    case BASS_OK: return "ok";
    case BASS_ERR_INVALID_ARG: return "invalid argument";
    case BASS_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case BASS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case BASS_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

// Draft-length heuristic, Algorithm 1 of the BASS paper (Section 3.2): grow when some sequence
// accepted every draft, otherwise shrink faster the longer the drafts are and the second time in
// a row, never below the largest accepted count.
extern "C" void bass_draft_len_init(bass_draft_len_state* state, int32_t l0) {
  if (!state) return;
  state->l_draft = l0 > 0 ? l0 : 7;
  state->s = 0;
}

extern "C" int32_t bass_next_draft_len(bass_draft_len_state* state, const int32_t* n_accept, int32_t B,
                                       int32_t l_incre, int32_t l_mod, int32_t l_limit) {
  if (!state || !n_accept || B <= 0 || state->l_draft <= 0) return BASS_ERR_INVALID_ARG;
  if (l_incre <= 0) l_incre = 2;
  if (l_mod <= 0) l_mod = 10;
  if (l_limit <= 0) l_limit = 32;
  int32_t most = n_accept[0];
  for (int32_t b = 1; b < B; ++b) most = n_accept[b] > most ? n_accept[b] : most;
  const int32_t l = state->l_draft;
  if (most == l) {
    state->l_draft = l + l_incre < l_limit ? l + l_incre : l_limit;
    state->s = 0;
  } else {
    int32_t next = l - (l + l_mod - 1) / l_mod - state->s;
    if (next < 1) next = 1;
    if (next < most) next = most;
    state->l_draft = next;
    state->s = 1;
  }
  return state->l_draft;
}
