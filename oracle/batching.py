"""CPU oracle (test infrastructure): the dynamic batching rule of PREBA section 4.3
("Dynamic Batching System for MIG") as a plain discrete-event simulation.

Single-input requests wait in one batching queue (the image path has one queue; the buckets
by input length are for audio).  Two parameters: Batch_max, the largest batch the system
builds, and Time_queue, the longest a request waits for its batch to be formed.  The rule as
read here: a batch is released as soon as Batch_max requests wait or the oldest has waited
Time_queue; it starts on the consumer (vGPU) that is free first, at that moment if one is
free, else when one becomes free; it is made of the oldest requests waiting at its start, at
most Batch_max.  Times are integers (nanoseconds).

Only tests and the benchmark's comparison leg may import this module.
"""

INF = 1 << 62


def time_queue_for(tail_knee, n_consumers):
    """Time_queue = (tail latency at the knee of one consumer) / (number of consumers)
    (section 4.3, "Analytical model based estimation for Time_queue")."""
    return tail_knee // n_consumers


def simulate(arrivals, n_consumers, batch_max, time_queue, service_time):
    """arrivals: non-decreasing integer times of requests 0..N-1; service_time(k): how long a
    consumer is busy with a batch of k.  Returns [(start, consumer, [request numbers])]."""
    n = len(arrivals)
    nxt = 0                      # next request that has not arrived yet
    queue = []                   # waiting requests, oldest first
    free = [0] * n_consumers     # when each consumer is free again
    batches = []
    while nxt < n or queue:
        if not queue:
            queue.append(nxt)
            nxt += 1
            continue
        # when the rule releases the next batch: the arrival that fills it, or the time limit
        # of the oldest request, whichever comes first
        if len(queue) >= batch_max:
            filled = arrivals[queue[batch_max - 1]]
        else:
            k = nxt + (batch_max - len(queue)) - 1
            filled = arrivals[k] if k < n else INF
        due = min(filled, arrivals[queue[0]] + time_queue)
        consumer = min(range(n_consumers), key=lambda c: (free[c], c))
        start = max(due, free[consumer])
        # whoever has arrived by then waits in the queue too
        while nxt < n and arrivals[nxt] <= start:
            queue.append(nxt)
            nxt += 1
        batch, queue = queue[:batch_max], queue[batch_max:]
        batches.append((start, consumer, batch))
        free[consumer] = start + service_time(len(batch))
    return batches
