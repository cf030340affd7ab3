"""The accesses one ef_moe_ffn call makes to the expert cache, replayed on the reference model
(oracle/lru_model.py): test plumbing shared by the CPU and GPU cache tests."""


def replay_layer(model, layer, need):
    """`need`: the experts the layer uses, in ascending id.  Resident ones are touched and pinned; misses that
    find a slot start at once; then everything held is released and the misses that found none take slots in
    waves (each wave holds its slots until its groups have run).  Ends with the clock tick of the layer."""
    held = []
    for e in need:
        if model.resident(layer, e):
            model.touch(layer, e)
            model.pin(layer, e)
            held.append(e)
    deferred = []
    for e in need:
        if e in held:
            continue
        if model.swap_in(layer, e, 0) == "busy":
            deferred.append(e)
            continue
        model.touch(layer, e)
        model.pin(layer, e)
        held.append(e)
    for e in held:
        model.pin(layer, e, False)
    while deferred:
        wave = []
        while deferred and model.swap_in(layer, deferred[0], 0) != "busy":
            e = deferred.pop(0)
            model.touch(layer, e)
            model.pin(layer, e)
            wave.append(e)
        assert wave, "no slot can be freed"
        for e in wave:
            model.pin(layer, e, False)
    model.advance(layer_run=layer)
