// HIP kernels of the RegTop-k round for gfx950 (wave64).
//
// Data flow of one round (all N workers batched; rows of length d):
//
//   k_begin         reset counters, load this round's speculative bound and window
//                   (only after a start without history: otherwise the compaction
//                   of the round before has prepared the control blocks)
//   k_accum_emit    a = eps + g written over eps (the one dense read/write sweep);
//                   eps is taken as 0 where the previous round's mask bit is set
//                   (the sent entries are never zeroed in memory: one bit per
//                   entry is read here instead of k scattered writes per worker);
//                   entries with |a| >= tau_lo are appended, in index order per
//                   4096-entry chunk, to the worker's candidate list
//   k_score         exact score of every candidate (regulariser for entries sent in
//                   the previous round; the value sent then travels with the
//                   candidate: the sweep finds it in the state it overwrites);
//                   scores inside a narrow window around the expected
//                   k-th score are also copied to a short boundary list, those
//                   above it are counted
//   k_select        one block per worker: checks the speculation (no overflow and
//                   >= k candidates scored >= tau_lo), then finds the k-th largest
//                   score exactly by a three-level radix select - over the boundary
//                   list when the window contains it, otherwise over all
//                   candidates - and derives next round's bound/window
//   (k_sample_hist, k_sample_bound: a round without history - round 0, after a
//                   reset - first takes its bound from a sample of a: whole
//                   128-byte lines at a fixed stride)
//   k_dense_all     for workers whose speculation failed: exact radix select of
//                   the k + k_prev largest priors |a|^y (k_prev entries were sent
//                   in the previous round, normally k; a superset of the true
//                   top-k, see below), count, scan and an ordered emission of
//                   exactly those entries as the candidate list, then their
//                   scores and the exact k-th score; one kernel with grid
//                   barriers between its phases, which returns at once when no
//                   worker is flagged
//   k_chunk_count / k_compact
//                   ordered compaction of the selected (index, value) pairs,
//                   lowest-index ties first: per-chunk counts of scores above and
//                   at the k-th, then placement from two levels of running sums;
//                   writes the round's mask (1 bit per entry)
//   k_aggregate     per 4096-entry tile: LDS accumulation of w*value in ascending
//                   worker order, tile written once (zero fill included)
//
// Why the k + k_prev largest priors suffice when the speculation fails: the
// score never exceeds the prior p = |a|^y (y = 1 unless a variant is set) and
// differs from it only on the k_prev entries sent in the previous round; among
// the k + k_prev entries with the largest (p, lower index first) at least k are
// therefore scored at their full p, and each of them beats every entry outside
// that set.
#pragma once
#include "common.h"
#include "sweep.h"
#include "score.h"
#include "select.h"
#include "dense.h"
#include "compact.h"
#include "extras.h"
