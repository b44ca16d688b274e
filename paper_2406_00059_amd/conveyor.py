"""Host-side tool-aware serving loop on top of the engine's per-token callback.

This is the part of the paper that sits above the engine (sections 3.2 and 3.3): tool developers wrap a tool
in a plugin that says when it can start and which pieces of decoded data it consumes; a streaming parser
turns the token stream into completed pieces as they are decoded; a token-granularity scheduler runs the LLM
one iteration at a time, hands every new token to the parser, starts a tool in a separate process as soon as
its plugin says it can start (tool partial execution), polls the running tools every iteration, and prefills
a tool's observation into the sequence when it is available.  With `partial=False` the same code is the
baseline of section 4.1: a tool starts only when its round has been decoded to the end.

While a request waits for its tool, its KV cache can stay on the GPU, be swapped to host memory, or be
discarded and recomputed (the options section 2.2 describes for systems that manage the cache across tool
calls); `retention` selects one, or lets `choose_retention` pick by the predicted tool time.

Everything here is host logic: no GPU work happens in this file, the engine does it.  Tools run in child
processes with a duplex pipe (section 3.3 steps (6), (7)); the children never touch the GPU.  They are forked
from a fork server, a single-threaded helper process, not from the serving process itself: that one holds the
GPU runtime's threads, and a child forked while one of them holds a lock could wait for it forever.  Call
start_tool_server() once before the first GPU call (it is started on first use otherwise).
"""
from __future__ import annotations

import multiprocessing as mp
import os
import time
from dataclasses import dataclass, field


# ------------------------------------------------------------------ parser

class StreamParser:
    """Streaming token parser: tokens in, completed pieces out.

    A piece is the run of tokens up to (not including) a delimiter; it is emitted at once when its delimiter
    is decoded.  `is_delimiter(token, index)` gets the token and its index inside the round, so synthetic
    workloads can place delimiters by position (a stand-in for a newline or a closing-quote token)."""

    def __init__(self, is_delimiter):
        self.is_delimiter = is_delimiter
        self.cur, self.index, self.pieces = [], 0, []

    def feed(self, token: int):
        done = []
        if self.is_delimiter(token, self.index):
            done.append(self.cur)
            self.pieces.append(self.cur)
            self.cur = []
        else:
            self.cur.append(token)
        self.index += 1
        return done

    def flush(self):
        """End of the round: the unterminated tail is the last piece."""
        if self.cur:
            self.pieces.append(self.cur)
            self.cur = []
        return self.pieces


# ------------------------------------------------------------------ plugin interface

class ToolPlugin:
    """What a tool developer writes: when the tool can start and what it does with the decoded pieces.

    `pieces_to_start` completed pieces are enough to start the tool (1: the invocation indicator, e.g. a
    function name; more: the indicator plus arguments; None: the tool needs the whole round).  `run` is
    executed in the tool's own process and returns the observation as token ids."""

    name = "tool"
    pieces_to_start = 1

    def can_start(self, pieces) -> bool:
        return self.pieces_to_start is not None and len(pieces) >= self.pieces_to_start

    def run(self, pieces):
        raise NotImplementedError


class SyntheticTool(ToolPlugin):
    """A tool of a set duration that returns a fixed, seeded observation."""

    def __init__(self, duration_s: float, observation, pieces_to_start=1, name="synthetic"):
        self.duration_s, self.observation = duration_s, [int(t) for t in observation]
        self.pieces_to_start, self.name = pieces_to_start, name

    def run(self, pieces):
        time.sleep(self.duration_s)
        return self.observation


def _tool_main(conn, plugin):
    try:
        pieces = conn.recv()
        t0 = time.perf_counter()
        obs = plugin.run(pieces)
        conn.send((obs, time.perf_counter() - t0))
    finally:
        conn.close()
        os._exit(0)          # no interpreter tear-down in the child: it shares nothing it may clean up


class _NoTool(ToolPlugin):
    def run(self, pieces):
        return []


_tool_ctx = None


def start_tool_server():
    """Starts the fork server that tool instances are forked from and runs one empty tool through it, so that
    the first real tool does not pay for the server's start.  Call it before the first GPU call of the
    process; later calls return at once.  Plugins travel to their process by pickle."""
    global _tool_ctx
    if _tool_ctx is None:
        ctx = mp.get_context("forkserver")
        ctx.set_forkserver_preload([__name__])
        _tool_ctx = ctx
        ToolProcess(_NoTool(), []).wait()
    return _tool_ctx


class ToolProcess:
    """One tool instance in a child process of the fork server, duplex pipe for the command and the observation."""

    def __init__(self, plugin: ToolPlugin, pieces):
        ctx = start_tool_server()
        self.started = time.perf_counter()
        self.conn, child = ctx.Pipe(duplex=True)
        self.proc = ctx.Process(target=_tool_main, args=(child, plugin), daemon=True)
        self.proc.start()
        child.close()
        self.conn.send(pieces)

    def kill(self):
        """Ends a tool that is given up on (time-out, aborted request)."""
        if self.proc.is_alive():
            self.proc.kill()
        self.proc.join()
        self.conn.close()

    def poll(self):
        """(observation, tool seconds) if the tool has finished, else None.  Never blocks."""
        if self.conn.poll(0):
            res = self.conn.recv()
            self.proc.join()
            return res
        return None

    def wait(self):
        res = self.conn.recv()
        self.proc.join()
        return res


# ------------------------------------------------------------------ requests and the scheduler

@dataclass
class Round:
    n_tokens: int                     # tokens generated in this round (the first comes from the prefill)
    tool: ToolPlugin | None = None    # tool invoked by this round's output (None: final round)
    delimiter_every: int = 8          # synthetic syntax: every k-th token of the round closes a piece


@dataclass
class Request:
    prompt: list
    rounds: list
    # filled in by the scheduler
    tokens: list = field(default_factory=list)        # all generated tokens
    g: list = field(default_factory=list)             # generation seconds per round (prefill + decode)
    t: list = field(default_factory=list)             # tool seconds per round (as measured in the child)
    s: list = field(default_factory=list)             # seconds into the round at which the tool was started
    retained: list = field(default_factory=list)      # per tool wait: "keep" | "swap" | "discard" | None (no wait)
    latency: float = 0.0
    failed: str | None = None                         # why the request was given up ("tool time-out ..."), else None


def choose_retention(ctx_tokens, tool_s, kv_bytes_per_token, swap_bytes_per_s, prefill_tokens_per_s):
    """What to do with the cache of a request that is about to wait `tool_s` seconds for its tool, by the
    GPU memory it wastes (bytes x seconds held without being read), as in the systems section 2.2 cites:
      keep:    M * tool_s                                  M = ctx_tokens * kv_bytes_per_token
      swap:    M * (2 M / swap_bytes_per_s)               held during the copy out and the copy back;
                                                          only if the copy out fits into the wait
      discard: M * (ctx_tokens / prefill_tokens_per_s)    held while it is being recomputed
    The smallest wins; ties go to the earlier entry."""
    M = ctx_tokens * kv_bytes_per_token
    t_copy = M / swap_bytes_per_s
    cost = {"keep": M * tool_s, "discard": M * (ctx_tokens / prefill_tokens_per_s)}
    if t_copy <= tool_s:
        cost["swap"] = M * 2 * t_copy
    order = ["keep", "swap", "discard"]
    return min((k for k in order if k in cost), key=lambda k: (cost[k], order.index(k)))


class Scheduler:
    """Token-granularity scheduler (section 3.3).  `engine` provides
         new_sequence() -> seq, prefill(seq, tokens) -> token, decode(seqs) -> tokens, free(seq)."""

    def __init__(self, engine, partial=True, retention="keep", predict_tool_s=None, rates=None, shared_prefix=0,
                 trim=False, tool_timeout_s=None):
        """retention: "keep" | "swap" | "discard" | "auto".  "auto" asks choose_retention with
        predict_tool_s(plugin) seconds and rates = dict(kv_bytes_per_token, swap_bytes_per_s,
        prefill_tokens_per_s).  "swap" needs engine.swap_out / engine.swap_in.
        shared_prefix = k > 0: all prompts start with the same k tokens (system prompt, tool descriptions);
        they are prefilled once and every request forks from that cache (engine.fork).
        trim: after every prefill (prompt or observation) the sequence gives up the cache blocks below its
        attention band (engine.trim; models with a band only).
        tool_timeout_s: a tool that has not answered that long after its start is killed and its request ends
        as failed (its cache is freed, the other requests go on); None: wait for ever."""
        self.engine, self.partial, self.retention, self.trim = engine, partial, retention, trim
        self.tool_timeout_s = tool_timeout_s
        self.predict_tool_s, self.rates, self.shared_prefix = predict_tool_s, rates or {}, shared_prefix

    def serve(self, requests):
        eng = self.engine
        t_start = time.perf_counter()
        st = []
        k, template = self.shared_prefix, None
        if k and requests:
            head = list(requests[0].prompt[:k])
            assert all(list(r.prompt[:k]) == head and len(r.prompt) > k for r in requests), "prompts must share the prefix"
            template = eng.new_sequence()
            eng.prefill(template, head)               # its emitted token is not used
        for r in requests:
            seq = eng.fork(template, k) if template is not None else eng.new_sequence()
            st.append(dict(req=r, seq=seq, round=0, left=0, parser=None, tool=None, obs=None,
                           feed=list(r.prompt[k:] if template is not None else r.prompt), round_t0=t_start,
                           t_start=t_start, done=False,
                           history=list(r.prompt[:k]) if template is not None else [], away=None, plugin=None))
        if template is not None:
            eng.free(template)                        # the shared blocks live on with their holders
        while not all(x["done"] for x in st):
            # (8) poll the plugins: collect observations of tools that have finished
            for x in st:
                if x["tool"] is not None and x["obs"] is None:
                    res = x["tool"].poll()
                    if res is not None:
                        x["obs"] = res
                    elif self.tool_timeout_s is not None and time.perf_counter() - x["tool"].started > self.tool_timeout_s:
                        x["tool"].kill()
                        x["req"].failed = f"tool time-out after {self.tool_timeout_s} s in round {x['round'] - (x['left'] == 0)}"
                        x["req"].latency = time.perf_counter() - x["t_start"]
                        if x["away"] == "swap":
                            eng.swap_in(x["seq"])     # the handle has to hold its blocks again to be freed like any other
                        if x["away"] != "discard":
                            eng.free(x["seq"])
                        x["tool"], x["done"], x["freed"] = None, True, True
            # (2) prefill whatever is ready: a new prompt, or an observation whose round has ended
            decoding = []
            for x in st:
                if x["done"]:
                    continue
                if x["feed"] is None and x["left"] == 0 and x["tool"] is not None and x["obs"] is not None:
                    obs, tool_s = x["obs"]
                    x["req"].t.append(tool_s)
                    x["feed"], x["tool"], x["obs"] = list(obs), None, None
                    x["round_t0"] = time.perf_counter()
                    if x["away"] == "swap":
                        eng.swap_in(x["seq"])
                    elif x["away"] == "discard":      # recompute: everything fed or generated so far, then the observation
                        x["seq"] = eng.new_sequence()
                        x["feed"] = x["history"] + x["feed"]
                        x["history"] = []
                    x["away"] = None
                elif (x["feed"] is None and x["left"] == 0 and x["tool"] is not None and x["obs"] is None
                      and x["away"] is None and not x["done"]):
                    x["away"] = self._retain(x)       # the round is over and its tool still runs
                if x["feed"] is not None:
                    rd = x["req"].rounds[x["round"]]
                    x["parser"] = StreamParser(lambda tok, i, k=rd.delimiter_every: (i + 1) % k == 0)
                    x["left"] = rd.n_tokens
                    x["history"].extend(x["feed"])
                    self._emit(x, eng.prefill(x["seq"], x["feed"]))
                    x["feed"] = None
                    if self.trim:                     # blocks that fell out of the attention band go back to the pool
                        eng.trim(x["seq"])
                elif x["left"] > 0:
                    decoding.append(x)
            # (2)+(3) one decoding iteration for every sequence that is generating; tokens go to the parsers
            if decoding:
                for x, tok in zip(decoding, eng.decode([x["seq"] for x in decoding])):
                    self._emit(x, tok)
            elif not any(x["feed"] is not None for x in st if not x["done"]):
                time.sleep(0.0005)       # every live request waits for a tool: nothing to run on the GPU
        for x in st:
            if not x.get("freed"):
                eng.free(x["seq"])
        return requests

    def _retain(self, x):
        """Called once per tool wait, when the round has been decoded and the observation is not there yet."""
        how = self.retention
        if how == "auto":
            how = choose_retention(len(x["history"]), self.predict_tool_s(x["plugin"]), **self.rates)
        if how == "swap":
            self.engine.swap_out(x["seq"])
        elif how == "discard":
            self.engine.free(x["seq"])
        x["req"].retained.append(how)
        return how

    def _emit(self, x, tok):
        req, rd = x["req"], x["req"].rounds[x["round"]]
        req.tokens.append(tok)
        x["history"].append(tok)
        x["left"] -= 1
        x["parser"].feed(tok)
        now = time.perf_counter()
        last = x["left"] == 0
        # (4)-(6): start the tool as soon as its plugin can start (partial execution), or at the end of the
        # round (baseline, and tools that need the whole output)
        if rd.tool is not None and x["tool"] is None:
            pieces = x["parser"].pieces
            if (self.partial and rd.tool.can_start(pieces)) or last:
                if last:
                    pieces = x["parser"].flush()
                x["tool"] = ToolProcess(rd.tool, [list(p) for p in pieces])
                x["plugin"] = rd.tool
                req.s.append(now - x["round_t0"])
        if last:
            req.g.append(now - x["round_t0"])
            if rd.tool is None:                       # final round: the response is ready (9)
                x["done"] = True
                req.latency = now - x["t_start"]
            else:
                x["round"] += 1


def serve(engine, requests, partial=True, **kw):
    """Runs the requests to completion; every request gets its tokens, per-round g / t / s and its latency
    (from the start of the call to its final token)."""
    return Scheduler(engine, partial, **kw).serve(requests)


# ------------------------------------------------------------------ engines

class LdEngine:
    """Adapter of the C-ABI engine to the scheduler's interface (argument marshalling only)."""

    def __init__(self, ld, kv_handle, stream=None):
        self.ld, self.kv, self.stream = ld, kv_handle, stream
        self._last, self._host, self._done = {}, {}, []

    def _cb(self, seq, tok, pos):
        self._last[seq] = tok
        return 0

    def new_sequence(self):
        return self.ld.ld_kv_alloc(self.kv, 0)

    def prefill(self, seq, tokens):
        self.ld.ld_prefill(self.kv, seq, tokens, self.stream, self._cb)   # returns after its tokens reached the host
        self._done.clear()                            # so every copy enqueued before it has finished
        return self._last[seq]

    def decode(self, seqs):
        self.ld.ld_decode_step(self.kv, seqs, self.stream, self._cb)
        return [self._last[s] for s in seqs]

    def free(self, seq):
        self._host.pop(seq, None)
        self.ld.ld_kv_free(self.kv, seq)

    def fork(self, parent, n_tokens):
        return self.ld.ld_kv_fork(self.kv, parent, n_tokens, self.stream)

    def trim(self, seq):
        """Sliding-window memory: give up the blocks below the attention band (nothing without a band)."""
        return self.ld.ld_kv_trim(self.kv, seq)

    def swap_out(self, seq):
        import torch                                  # pinned host memory only
        buf = torch.empty(max(self.ld.ld_kv_swap_bytes(self.kv, seq), 1), dtype=torch.uint8, pin_memory=True)
        self.ld.ld_kv_swap_out(self.kv, seq, buf, self.stream)
        self._host[seq] = buf                         # stays alive until the copy back has been enqueued and run

    def swap_in(self, seq):
        self.ld.ld_kv_swap_in(self.kv, seq, self._host[seq], self.stream)
        self._done.append(self._host.pop(seq))        # released by the next prefill's synchronisation
