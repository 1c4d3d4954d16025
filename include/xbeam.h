/*
 * Host-side beam-search selection step (section 4.5.1 "Host-side Optimization", paragraph "Beam Search
 * Optimization"): out of the beam_width * top_k candidate continuations of a request's beam_width
 * sequences, pick the beam_width best and return them in descending order of score.  Everything here
 * runs on the CPU: every pointer is a HOST pointer.  Same status codes and error text
 * (xattn_last_error) as xattn.h.
 */
#ifndef XBEAM_H_
#define XBEAM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* flags */
enum { XBEAM_FULL_SORT = 1,      /* baseline for comparison: score and sort all candidates, no heap, no early exit */
       XBEAM_CHECK_INPUT = 2 };  /* verify the precondition on cand_lp (costs a pass over all candidates) */

/*
 * Candidate (w, k) of request r has score beam_lp[r][w] + cand_lp[r][w][k], added in fp32.  The result
 * is the first beam_width candidates in the order "score descending, then w ascending, then k
 * ascending" (so it is unique, also among equal scores).
 *
 * Method: one min-heap of beam_width entries per request; the sequences are visited in order, each
 * one's candidates in order of k; a candidate that does not beat the heap's worst entry ends the visit
 * of its sequence, since cand_lp[r][w][:] is descending; finally the heap is emptied worst-first into
 * the output from the back.  No allocation after the first call on a thread (the heap is reused), and
 * the outputs are the caller's arrays.
 *
 * beam_lp   HOST fp32 [n_req, beam_width]         log-probability of each live sequence
 * cand_lp   HOST fp32 [n_req, beam_width, top_k]  log-probabilities of its top_k next tokens, DESCENDING
 *                                                 along the last axis; -inf allowed, NaN not
 * cand_tok  HOST int32 [n_req, beam_width, top_k] the tokens, or NULL (then out_tok receives k)
 * out_lp    HOST fp32 [n_req, beam_width]         scores of the selected candidates, descending
 * out_parent HOST int32 [n_req, beam_width]       w of each selected candidate
 * out_tok   HOST int32 [n_req, beam_width]        its token
 * visited   HOST int64 [n_req] or NULL            candidates examined (beam_width * top_k without early exit)
 * Outputs must not overlap inputs.  n_req >= 0, 1 <= beam_width <= 65536, 1 <= top_k <= 65536.
 * Returns XATTN_OK, or XATTN_EINVAL (bad sizes, NULL, or, with XBEAM_CHECK_INPUT, an ascending step or a
 * NaN in cand_lp / beam_lp) with nothing written for the offending request and those after it.
 */
int xbeam_select(const float* beam_lp, const float* cand_lp, const int32_t* cand_tok, int n_req, int beam_width,
                 int top_k, int flags, float* out_lp, int32_t* out_parent, int32_t* out_tok, int64_t* visited);

#ifdef __cplusplus
}
#endif
#endif
