"""Writes two_key_sigmoid.json: logistic values to 30 digits from the decimal module only."""
import json
import os
from decimal import Decimal, getcontext

getcontext().prec = 50
gaps = ["0.5", "1", "2", "8"]          # score gaps that bf16 inputs can realise exactly
rows = [{"gap": g, "sigmoid": str(+(1 / (1 + (-Decimal(g)).exp())).quantize(Decimal(10) ** -30))}
        for g in gaps]
with open(os.path.join(os.path.dirname(__file__), "two_key_sigmoid.json"), "w") as f:
    json.dump({"identity": "softmax([0, gap]) = [1 - sigmoid(gap), sigmoid(gap)]", "rows": rows}, f, indent=1)
