"""Seeded synthetic request traces with the structure of the paper's workloads (Section 5.1, "Workloads":
multi-turn chat sessions whose rounds append to the conversation so far; Section 4.1: prompts shared by many
requests, i.e. system prompts and few-shot examples).  The datasets themselves are not available; only the shape is
kept: a few shared prompt prefixes, sessions that start from one of them, rounds whose input is the whole history
plus new user tokens, outputs of random length, sessions interleaved in arrival order.  Token ids are random
integers; nothing here is text.

Only random draws happen here; no cache logic.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def make_trace(seed: int, n_sessions: int = 12, n_prompts: int = 3, prompt_len=(20, 60), turns=(1, 5),
               user_len=(3, 25), out_len=(2, 30), vocab: int = 1000) -> List[Tuple[List[int], List[int]]]:
    """Returns requests in arrival order as (input tokens, output tokens)."""
    rs = np.random.RandomState(seed)
    prompts = [list(map(int, rs.randint(0, vocab, size=rs.randint(prompt_len[0], prompt_len[1] + 1))))
               for _ in range(n_prompts)]
    sessions = []
    for _ in range(n_sessions):
        rounds = []
        history = list(prompts[rs.randint(n_prompts)])
        for _ in range(rs.randint(turns[0], turns[1] + 1)):
            user = list(map(int, rs.randint(0, vocab, size=rs.randint(user_len[0], user_len[1] + 1))))
            out = list(map(int, rs.randint(0, vocab, size=rs.randint(out_len[0], out_len[1] + 1))))
            inp = history + user
            rounds.append((inp, out))
            history = inp + out
        sessions.append(rounds)
    # interleave: repeatedly pick a session that still has rounds left
    trace = []
    cursors = [0] * n_sessions
    live = [i for i in range(n_sessions)]
    while live:
        i = live[rs.randint(len(live))]
        trace.append(sessions[i][cursors[i]])
        cursors[i] += 1
        if cursors[i] == len(sessions[i]):
            live.remove(i)
    return trace


def make_mixed_trace(seed: int, n_docs: int = 6, doc_len=(3000, 9000), n_requests: int = 1500, p_doc: float = 0.25,
                     chat_len=(50, 600), q_len=(20, 100), out_len=(20, 200),
                     vocab: int = 32000) -> List[Tuple[List[int], List[int]]]:
    """Long shared documents queried again and again (the "purely input" prefixes of Section 4.1: long-document QA,
    few-shot prompts) among many short one-off chats that are never reused: the mix in which recency alone throws
    away the entries that save the most compute per byte (Section 4.2)."""
    rs = np.random.RandomState(seed)
    docs = [list(map(int, rs.randint(0, vocab, size=rs.randint(doc_len[0], doc_len[1] + 1)))) for _ in range(n_docs)]
    trace = []
    for _ in range(n_requests):
        if rs.rand() < p_doc:
            inp = docs[rs.randint(n_docs)] + list(map(int, rs.randint(0, vocab, size=rs.randint(q_len[0], q_len[1] + 1))))
        else:
            inp = list(map(int, rs.randint(0, vocab, size=rs.randint(chat_len[0], chat_len[1] + 1))))
        trace.append((inp, list(map(int, rs.randint(0, vocab, size=rs.randint(out_len[0], out_len[1] + 1))))))
    return trace
