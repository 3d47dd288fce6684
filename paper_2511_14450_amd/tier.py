"""One tier of the pipeline as several replicas of a stage on one device: the node set
K_j of Sec. IV-B.  Every replica ("node") owns a HIP stream, which is its FIFO task
queue Q_{j,k}: a task's prefill and decode steps are enqueued behind whatever the node
already holds.  An arriving task is given to the node HypSched-RT (Algorithm 2, the
library's `hypsched_rt`) picks from the nodes' queue state: the remaining workload of
the running task plus the workloads waiting, over the node's capacity.

Only bookkeeping happens here; the blocks run in the HIP library and the choice is the
library's.  Run as a program it replays a Poisson arrival stream (Sec. V-A models
arrivals with lambda = 0.2 tasks / s; the rate is a parameter because one MI355X serves
such a stream without ever queueing) and prints per-task latencies next to what the
queue model `hypsched_simulate` predicts from the measured service time.

    python -m paper_2511_14450_amd.tier --nodes 3 --tasks 14 --rate 40
"""
from __future__ import annotations

import argparse
import json
import time
from typing import Callable, Dict, List, Optional, Sequence

import torch

from . import binding


class _Task:
    __slots__ = ("work", "mem", "pred_finish", "done", "out", "t_submit", "node")

    def __init__(self, work, mem, pred_finish, done, out, t_submit, node):
        self.work, self.mem, self.pred_finish, self.done = work, mem, pred_finish, done
        self.out, self.t_submit, self.node = out, t_submit, node


class Tier:
    """n_nodes replicas of the stage over blocks [l_start, l_end).

    capacity[k]   C_{j,k}: work per second node k is credited with (1.0 = a task of
                  workload F takes F seconds); replicas on one device are equal, the
                  parameter exists so that tests can make the scheduler's choice visible
    memory[k]     M_{j,k}: what the node can hold in the unit of a task's m_act
    """

    def __init__(self, shape, l_start: int, l_end: int, layer_fn: Callable[[int], Dict[str, torch.Tensor]],
                 n_nodes: int, max_batch: int, max_seq: int, max_prefill_tokens: int,
                 capacity: Optional[Sequence[float]] = None, memory: Optional[Sequence[float]] = None, flags: int = 0):
        if n_nodes < 1:
            raise ValueError("a tier needs at least one node")
        self.capacity = [1.0] * n_nodes if capacity is None else [float(c) for c in capacity]
        self.memory = [float("inf")] * n_nodes if memory is None else [float(v) for v in memory]
        if len(self.capacity) != n_nodes or len(self.memory) != n_nodes:
            raise ValueError("capacity / memory need one entry per node")
        self.available = [True] * n_nodes
        self.streams = [torch.cuda.Stream() for _ in range(n_nodes)]
        self.stages: List[binding.Stage] = []
        layers = [layer_fn(l) for l in range(l_start, l_end)]
        for k in range(n_nodes):
            cfg = binding.stage_config(shape, max_batch, max_seq, max_prefill_tokens, flags)
            with torch.cuda.stream(self.streams[k]):
                self.stages.append(binding.stage_create(cfg, l_start, l_end, layers, stream=self.streams[k]))
        del layers
        torch.cuda.synchronize()
        self.queues: List[List[_Task]] = [[] for _ in range(n_nodes)]
        self.decisions: List[dict] = []  # what the scheduler saw and chose, task by task

    def node_state(self, now: float):
        """(M_avail, F_run_rem, F_wait) per node at host time `now`; completed tasks leave."""
        M_avail, F_run, F_wait = [], [], []
        for k, q in enumerate(self.queues):
            while q and q[0].done.query():
                q.pop(0)
            used = sum(t.mem for t in q)
            M_avail.append(self.memory[k] - used)
            F_run.append(max(0.0, q[0].pred_finish - now) * self.capacity[k] if q else 0.0)
            F_wait.append(sum(t.work for t in q[1:]))
        return M_avail, F_run, F_wait

    def submit(self, hidden: torch.Tensor, seq_lens: Sequence[int], decode_steps: int, work: float,
               mem: float = 0.0) -> Optional[_Task]:
        """A task: prefill of `hidden` ([sum seq_lens, H]) and `decode_steps` steps, each fed
        the stage's previous output for the requests' last positions.  `work` is its F_j*
        (seconds on a node of capacity 1), `mem` its m_act.  Returns None if HypSched-RT
        finds no eligible node (the caller decides whether to retry)."""
        now = time.perf_counter()
        M_avail, F_run, F_wait = self.node_state(now)
        k = binding.hypsched_rt(work, mem, self.capacity, M_avail, self.available, F_run, F_wait)
        self.decisions.append(dict(F_new=work, m_act=mem, C=list(self.capacity), M_avail=M_avail,
                                   available=list(self.available), F_run_rem=F_run, F_wait=F_wait, k=k))
        if k is None:
            return None
        q = self.queues[k]
        start = max(now, q[-1].pred_finish) if q else now
        stage, stream = self.stages[k], self.streams[k]
        stream.wait_stream(torch.cuda.current_stream())  # the caller's tensor is ready on its stream
        with torch.cuda.stream(stream):
            out = binding.stage_prefill(stage, hidden, seq_lens)
            if decode_steps:
                ends = torch.cumsum(torch.tensor(list(seq_lens)), 0) - 1
                h = out[ends.to(out.device)].contiguous()
                for _ in range(decode_steps):
                    h = binding.stage_decode_step(stage, h)
                out = h
            done = torch.cuda.Event()
            done.record(stream)
        hidden.record_stream(stream)
        task = _Task(work, mem, start + work / self.capacity[k], done, out, now, k)
        q.append(task)
        return task

    def destroy(self) -> None:
        torch.cuda.synchronize()
        for st in self.stages:
            st.destroy()
        self.stages = []


def main():
    from .chain import MODELS, _Shape, _synthetic_layer
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--model", choices=sorted(MODELS), default="phi3_medium")
    ap.add_argument("--blocks", type=int, default=7, help="blocks of the tier's stage (Table II gives tier 3 seven)")
    ap.add_argument("--nodes", type=int, default=3)
    ap.add_argument("--tasks", type=int, default=14)
    ap.add_argument("--rate", type=float, default=40.0, help="Poisson arrival rate, tasks per second")
    ap.add_argument("--prompt", type=int, default=64)
    ap.add_argument("--generate", type=int, default=128)
    ap.add_argument("--seed", type=int, default=251114450)
    a = ap.parse_args()
    m = MODELS[a.model]
    shape = _Shape(m)
    tier = Tier(shape, 0, a.blocks, _synthetic_layer(shape, a.seed), a.nodes, 1, a.prompt + a.generate + 1, a.prompt)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(a.seed + 11)
    xs = [torch.randn((a.prompt, m["hidden"]), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(a.tasks)]
    # service time of one task alone on an idle device: the F_j* every task is credited with
    for _ in range(2):
        t0 = time.perf_counter()
        t = tier.submit(xs[0], [a.prompt], a.generate - 1, 1.0)
        t.done.synchronize()
        service = time.perf_counter() - t0
    tier.decisions.clear()
    gcpu = torch.Generator().manual_seed(a.seed + 12)
    gaps = torch.empty(a.tasks).exponential_(a.rate, generator=gcpu).tolist()
    arrivals, acc = [], 0.0
    for g in gaps:
        acc += g
        arrivals.append(acc)
    tasks = []
    t_begin = time.perf_counter()
    for q in range(a.tasks):
        while time.perf_counter() - t_begin < arrivals[q]:
            time.sleep(0.0002)
        tasks.append(tier.submit(xs[q], [a.prompt], a.generate - 1, service))
    for t in tasks:
        t.done.synchronize()
    torch.cuda.synchronize()
    t_end = time.perf_counter() - t_begin
    nodes = [t.node for t in tasks]
    sim_nodes, sim_finish = binding.hypsched_simulate(arrivals, [service], [0.0], [[1.0] * a.nodes],
                                                      [[float("inf")] * a.nodes], [])
    res = {"workload": "one tier, Poisson arrivals, HypSched-RT over stage replicas on separate streams",
           "model": a.model, "blocks": a.blocks, "nodes": a.nodes, "tasks": a.tasks, "rate_per_s": a.rate,
           "service_s_alone": service, "makespan_s": t_end,
           "queue_model_makespan_s": max(f[0] for f in sim_finish),
           "nodes_chosen": nodes, "queue_model_nodes": [n[0] for n in sim_nodes]}
    print(json.dumps(res))
    tier.destroy()


if __name__ == "__main__":
    main()
